// 256 x 256-tile form of the fused hidden layer of Alg. 4 for large products:
// a^b_k = Sign(BatchNorm(XnorDotProduct(a^b_{k-1}, W^b_k))) (Sec. 4 Eq. (5)), bits in, bits out.
//
// Same arithmetic as xnor_gemm_mfma.hip (bits widened in registers to fp4 codes whose products are 1,
// v_mfma_f32_32x32x64_f8f6f4, exact fp32 sums S, pre-activation K - 2pa - 2pb + 4S, threshold folded into
// the sums by a rank-2 fp32 MFMA, output bit = complement of the sign), organised for ONE wavefront per
// SIMD: a workgroup of 4 wavefronts owns a 256 x 256 tile, each wavefront 4 x 4 accumulator blocks of
// 32 x 32 (256 accumulation registers; a wavefront alone on its SIMD has 512 registers).  A K-step of 64
// then widens 4 + 4 operand words for 16 MFMAs, 2.75 vector-ALU operations per MFMA against 4.0 for the
// 4 x 2 blocks of the two-wavefronts-per-SIMD kernels, whose K loop is limited by exactly that issue
// traffic.  With nothing else resident on the SIMD, latencies are hidden in the instruction stream itself:
//   - three LDS buffers of one K-tile (512 bits of K) each; K-tile t+2 is written while K-tile t is
//     multiplied, its global loads having been issued most of a K-tile earlier;
//   - one barrier per K-tile, in the middle of it, so that the LDS reads of the next K-tile's first
//     half are issued under the MFMAs of the second half of the current one;
//   - the operands of K-step s+1 are widened between the MFMAs of step s, every memory operation has a
//     slot after an MFMA of its own (BNN_STEP_SCHEDULE), the first K-step of a tile starts the sums with a
//     zero addend (no clearing of 256 registers);
//   - the stream of K-tiles runs on across the workgroup's output tiles: the first two K-tiles of the next
//     tile are in LDS when the current tile's epilogue starts.
// Work split: one workgroup per compute unit.  The N / 256 column tiles times `strips` row strips are the
// workgroups; a strip's rows are covered by 256-row tiles and, where at most 128 rows remain, one 128-row
// tile (2 x 4 blocks per wavefront), the last tile shifted up to end with the strip (shared rows are
// computed and written twice with the same values).  Every compute unit gets the same number of rows, which
// is what a grid of whole tiles cannot do when the tile count is not a multiple of the compute units
// (M = 10000, N = 4096: 640 tiles on 256 compute units = 3 rounds; here 2 tiles and a half tile each).
// Takes only products where nothing has to be checked per element (the launcher refuses the rest):
// K a multiple of 512 with 2048 <= K <= kMfmaFoldMaxK, N a multiple of 256 whose tile count divides the
// compute units, strips of at least 256 rows, operands that allow 16-byte loads, leading dimensions below
// 2^22 words, output rows that allow 8-byte stores.
#include <type_traits>

#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {

namespace big {

constexpr int WN = 4;                              // accumulator blocks per wavefront along N
constexpr int BN = 64 * WN;                        // 2 x 2 wavefronts: 256 columns
constexpr int BM_MAX = 256;                        // rows of the large tile (4 blocks per wavefront along M)
constexpr int PLANE = BM_MAX + 2;                  // 16-byte slots per quad plane (2 pad slots)
constexpr int BUF = kMfmaKQ * PLANE;               // slots of one operand's K-tile
constexpr int NBUF = 3;
constexpr int ST_ROWS = 256 / kMfmaKQ;             // rows covered by one staging pass
constexpr int LOADS_B = BN / ST_ROWS;              // staging passes of B
static_assert(BN == BM_MAX && kMfmaKQ == 4, "square large tile, 4 staging lanes per row");

typedef int v4i __attribute__((ext_vector_type(4)));

// The four fp4 operand registers of a word (see widen_fp4_a / widen_fp4_b); the MFMA's operand type has
// eight, of which the fp4 format reads four.
__device__ inline v4i widen4_a(uint32_t w) {
    return v4i{int(w & 0x11111111u), int(w & 0x22222222u), int(w & 0x44444444u), int((w >> 2) & 0x22222222u)};
}
__device__ inline v4i widen4_b(uint32_t w) {
    const uint32_t r = w >> 2;
    return v4i{int((w << 2) & 0x44444444u), int(w & 0x22222222u), int(r & 0x11111111u), int(r & 0x22222222u)};
}
__device__ inline v8i operand8(v4i f) { return v8i{f[0], f[1], f[2], f[3], 0, 0, 0, 0}; }

__device__ inline uint4 load16_at(const uint32_t* uniform_base, uint32_t lane_byte_offset) {
    return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(uniform_base) + lane_byte_offset);
}

// What a workgroup shares in LDS.
struct Shared {
    uint4 a[NBUF * BUF];
    uint4 b[NBUF * BUF];
    float pop_af[BM_MAX];          // popcount(A row) / 2 of the tile whose row sums were published last
    int thr[BN];                   // the column tile's thresholds, clamped to [-K-1, K+1]
    uint32_t flip[BN / 32];
    float colfix[BN];              // fold_column_term of the column tile
};

// Fused epilogue on TRANSPOSED accumulator blocks (the MFMAs were issued with the operands swapped:
// register v of lane l is column 8*(v/4) + 4*(l/32) + v%4 and row l%32 of its block), as in
// mfma_output_words: the folded threshold is added by one rank-2 fp32 MFMA per block (exact for
// K <= kMfmaFoldMaxK), the output bit is the complement of the accumulator's sign, collected with
// v_alignbit.  The MFMAs of block row i + 1 are issued before the vector-ALU work on row i.  The
// wavefront's four column blocks are handled as the pairs (0, 2) and (1, 3): after the half swap lanes
// 0-31 hold the words of blocks 0 and 1, lanes 32-63 those of blocks 2 and 3, so each lane stores its
// row's two adjacent words with one 8-byte store.
template <int WM>
__device__ inline void epilogue_bits(v16f (&acc)[WM][WN], const Shared& sh, const BnSignArgs& bn, int row0,
                                     int col0, int wm, int wn, int fr, int fh) {
    const uint2 flip2 = make_uint2(sh.flip[wn * WN + 2 * fh], sh.flip[wn * WN + 2 * fh + 1]);
    float left[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) left[j] = fh == 0 ? sh.colfix[wn * 32 * WN + j * 32 + fr] : 1.0f;
    uint32_t* out_base = bn.out + (int64_t(row0 + wm * 32 * WM) * bn.ld_out + ((col0 + wn * 32 * WN) >> 5));   // uniform
    auto fold_row = [&](int i) {
        const float right = fh == 0 ? 1.0f : -sh.pop_af[wm * 32 * WM + i * 32 + fr];
        // In place: the kernel's 256 accumulation registers are all taken by the blocks.
#pragma unroll
        for (int j = 0; j < WN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(left[j], right, acc[i][j], 0, 0, 0);
    };
    fold_row(0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        if (i + 1 < WM) fold_row(i + 1);
        __builtin_amdgcn_sched_barrier(0);
        uint32_t part[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            // Sign bits of the block's 16 registers, nibble g (columns 8g + 4*fh ...) at bit 8g.
            uint32_t neg = 0u;
#pragma unroll
            for (int g = 3; g >= 0; --g) {
#pragma unroll
                for (int e = 3; e >= 0; --e)
                    neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[i][j][4 * g + e]), 31);
                if (g > 0) neg <<= 4;
            }
            part[j] = (~neg & 0x0F0F0F0Fu) << (4 * fh);
            // Keeps the accumulator reads of the blocks apart: read all at once they need more
            // registers than the K loop's state leaves free.
            __builtin_amdgcn_sched_barrier(0);
        }
        // Pair (0, 2): lanes 32-63 of part[0] <-> lanes 0-31 of part[2]; likewise (1, 3).
        const auto s02 = __builtin_amdgcn_permlane32_swap(part[0], part[2], false, false);
        const auto s13 = __builtin_amdgcn_permlane32_swap(part[1], part[3], false, false);
        const uint2 w = make_uint2((s02[0] | s02[1]) ^ flip2.x, (s13[0] | s13[1]) ^ flip2.y);
        *reinterpret_cast<uint2*>(out_base + (int64_t(i * 32 + fr) * bn.ld_out + 2 * fh)) = w;
    }
}

// Instruction order inside one K-step.  A wavefront alone on its SIMD keeps the matrix pipe busy (one
// MFMA per 32 cycles) only while the instructions between two MFMAs issue within those 32 cycles;
// measured, an MFMA takes about 8 of them, a vector-ALU operation about 5, and a 16-byte LDS write or
// global load holds the wavefront for 10 - 20.  So after every MFMA: at most one memory operation of the
// kind(s) KIND and at most VALU vector-ALU operations (the widening of the next K-step, the row
// popcounts).  Masks of __builtin_amdgcn_sched_group_barrier: 0x2 vector ALU, 0x8 MFMA, 0x20 global
// loads, 0x100 LDS reads, 0x200 LDS writes.  The closing sched_barrier(0) keeps the steps apart: without
// it the scheduler widens the operands of all later steps early and runs out of registers.
#define BNN_STEP_SCHEDULE(MFMAS, KIND, VALU)                               \
    do {                                                                   \
        _Pragma("unroll") for (int g_ = 0; g_ < (MFMAS); ++g_) {           \
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);             \
            __builtin_amdgcn_sched_group_barrier(KIND, 1, 0);              \
            __builtin_amdgcn_sched_group_barrier(0x002, VALU, 0);          \
        }                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                 \
    } while (0)

// The output tiles of `count` row tiles of 64 * WM rows each, at rows min(first_row + 64 * WM * i, last_row0)
// and columns [col0, col0 + 256), i = 0 .. count - 1 (count >= 1), n_ktiles >= 4.  The thresholds of the
// column tile are either in sh.thr / sh.flip, a barrier having been passed since they were written, or
// (write_thr) still in this thread's registers - thr_reg of column col0 + threadIdx.x, flip_reg of word
// threadIdx.x < 8 - and written here, once the first operand loads are under way: their first readers, the
// row sums of the first tile, are several barriers further on.
template <int WM>
__device__ inline void run_row_tiles(const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B,
                                     int64_t ldb, int K, const BnSignArgs& bn, Shared& sh, int first_row,
                                     int last_row0, int count, int col0, bool write_thr, int thr_reg,
                                     uint32_t flip_reg) {
    constexpr int BM = 64 * WM;
    constexpr int LOADS_A = BM / ST_ROWS;
    constexpr int MFMAS = WM * WN;                      // per K-step
    // Vector-ALU operations per MFMA slot: the widening of a K-step (5 per word of A, 6 per word of B)
    // spread over its MFMAs.
    constexpr int VALU = (5 * WM + 6 * WN + MFMAS - 1) / MFMAS;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;
    const int n_ktiles = K / (32 * kMfmaKT);
    const int st_q = tid % kMfmaKQ, st_r = tid / kMfmaKQ;
    const int st_slot = st_q * PLANE + st_r;                                      // + l * ST_ROWS + buffer
    const int rd_a = 2 * fh * PLANE + wm * 32 * WM + fr;                          // + hq * PLANE + i * 32 + buffer
    const int rd_b = 2 * fh * PLANE + wn * 32 * WN + fr;

    // Fetch cursor: row tile, K-tile and the two wavefront-uniform addresses (first word of the K-tile in
    // the tile's first row of A / B) of the next global loads.  It stops at the last K-tile of the last
    // tile, so that the (unconditional) loads always stay inside the operands.  A lane's loads are
    // `uniform address + its byte offset in staging pass l`: scalar base, one offset register each,
    // nothing to compute per load but one pointer step per K-tile.
    int f_tile = 0, f_kt = 0;
    const uint32_t* f_a = A + int64_t(min(first_row, last_row0)) * lda;
    const uint32_t* f_b = B + int64_t(col0) * ldb;
    auto advance_fetch = [&]() {
        if (__builtin_expect(f_kt + 1 < n_ktiles, 1)) {
            ++f_kt;
            f_a += kMfmaKT;
            f_b += kMfmaKT;
        } else if (f_tile + 1 < count) {
            f_kt = 0;
            ++f_tile;
            f_a = A + int64_t(min(first_row + BM * f_tile, last_row0)) * lda;
            f_b = B + int64_t(col0) * ldb;
        }
    };
    uint32_t a_lane[LOADS_A], b_lane[LOADS_B];          // byte offsets (leading dimensions < 2^22 words)
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) a_lane[l] = (uint32_t(st_r + l * ST_ROWS) * uint32_t(lda) + 4u * st_q) * 4u;
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) b_lane[l] = (uint32_t(st_r + l * ST_ROWS) * uint32_t(ldb) + 4u * st_q) * 4u;

    uint4 ra[LOADS_A], rb[LOADS_B];
    int cnt_a[LOADS_A], cnt_b[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) cnt_a[l] = 0;
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) cnt_b[l] = 0;

    // The lane offsets are made opaque at each use so that `uniform address + 32-bit lane offset` stays in
    // that form instead of becoming a 64-bit address per lane.
    auto fetch_a = [&](uint4 (&r)[LOADS_A]) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            uint32_t off = a_lane[l];
            asm volatile("" : "+v"(off));
            r[l] = load16_at(f_a, off);
        }
    };
    auto fetch_b = [&](uint4 (&r)[LOADS_B], const uint32_t* from) {
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            uint32_t off = b_lane[l];
            asm volatile("" : "+v"(off));
            r[l] = load16_at(from, off);
        }
    };
    // Set bits of a fetched quad added to a row sum, as a chain of popcount-and-add operations
    // (v_bcnt_u32_b32 adds its second operand; the empty asm statements keep the compiler from turning the
    // chain into four plain popcounts and two three-operand additions).
    auto add_bits = [](int c, const uint4& v) {
        c = __builtin_popcount(v.x) + c;
        asm("" : "+v"(c));
        c = __builtin_popcount(v.y) + c;
        asm("" : "+v"(c));
        c = __builtin_popcount(v.z) + c;
        asm("" : "+v"(c));
        return __builtin_popcount(v.w) + c;
    };
    // stage_a / stage_b write fetched words to LDS; count_a / count_b add their set bits to this thread's row sums.
    auto stage_a = [&](int buf, const uint4 (&r)[LOADS_A]) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) sh.a[buf * BUF + st_slot + l * ST_ROWS] = r[l];
    };
    auto stage_b = [&](int buf, const uint4 (&r)[LOADS_B]) {
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) sh.b[buf * BUF + st_slot + l * ST_ROWS] = r[l];
    };
    auto count_a = [&](const uint4 (&r)[LOADS_A]) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) cnt_a[l] = add_bits(cnt_a[l], r[l]);
    };
    auto count_b = [&](const uint4 (&r)[LOADS_B]) {
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) cnt_b[l] = add_bits(cnt_b[l], r[l]);
    };
    // Row sums of a finished tile: the 4 threads that staged the quads of one row are neighbouring lanes.
    // The epilogue needs popcount(A row) / 2 and, per column, fold_column_term(thr, K, 2 * popcount(B row)).
    auto publish_row_sums = [&]() {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            int c = cnt_a[l];
            c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);       // lane ^ 1
            c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);       // lane ^ 2
            if (st_q == 0) sh.pop_af[st_r + l * ST_ROWS] = 0.5f * float(c);
            cnt_a[l] = 0;
        }
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            int c = cnt_b[l];
            c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);
            c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);
            if (st_q == 0) sh.colfix[st_r + l * ST_ROWS] = fold_column_term(sh.thr[st_r + l * ST_ROWS], K, 2 * c);
            cnt_b[l] = 0;
        }
    };

    v16f acc[WM][WN];

    // The lane's words of a half K-tile: quad 2*fh + hq of each of its WM + 4 block rows; a quad feeds 4 K-steps.
    auto read_quads_a = [&](int buf, int hq, uint4 (&qa)[WM]) {
#pragma unroll
        for (int i = 0; i < WM; ++i) qa[i] = sh.a[buf * BUF + rd_a + hq * PLANE + i * 32];
    };
    auto read_quads_b = [&](int buf, int hq, uint4 (&qb)[WN]) {
#pragma unroll
        for (int j = 0; j < WN; ++j) qb[j] = sh.b[buf * BUF + rd_b + hq * PLANE + j * 32];
    };
    // Operands of the K-step that is multiplied next, widened one step ahead of their use so that the
    // widening of step s + 1 is issued between the MFMAs of step s.
    v4i fa[WM], fb[WN];
    auto widen_step = [&](const uint4 (&qa)[WM], const uint4 (&qb)[WN], int s, v4i (&oa)[WM], v4i (&ob)[WN]) {
#pragma unroll
        for (int i = 0; i < WM; ++i) oa[i] = widen4_a(quad_word(qa[i], s));
#pragma unroll
        for (int j = 0; j < WN; ++j) ob[j] = widen4_b(quad_word(qb[j], s));
    };
    // K-step: widens the operands of the next step (word s_next of the quads (na, nb)) and multiplies the
    // operands widened during the previous step.  first: the first K-step of an output tile, which
    // starts the sums (a zero addend instead of the accumulator).
    auto k_step = [&](const uint4 (&na)[WM], const uint4 (&nb)[WN], int s_next, auto first_tag) {
        constexpr bool FIRST = decltype(first_tag)::value;
        v4i xa[WM], xb[WN];
        widen_step(na, nb, s_next, xa, xb);
        // Literal zero scale operands select the plain v_mfma_f32_32x32x64_f8f6f4.  The operands are
        // swapped: the accumulator blocks are the transposes of the output blocks, so the epilogue can
        // pack a row's bits inside a lane.
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                v16f addend = acc[i][j];
                if (FIRST) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) addend[v] = 0.0f;
                }
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(operand8(fb[j]), operand8(fa[i]), addend, 4, 4, 0, 0, 0, 0);
            }
#pragma unroll
        for (int i = 0; i < WM; ++i) fa[i] = xa[i];
#pragma unroll
        for (int j = 0; j < WN; ++j) fb[j] = xb[j];
    };

    // Prologue: K-tiles 0 and 1 of the stream into LDS, A's part of K-tile 2 in flight.  The first two
    // are fetched together, the second into the registers of the quads.
    uint4 qa0[WM], qb0[WN], qa1[WM], qb1[WN];
    static_assert(WM == LOADS_A && WN == LOADS_B, "the prologue borrows the quad registers for a fetch");
    fetch_a(ra);
    fetch_b(rb, f_b);
    advance_fetch();
    fetch_a(qa0);
    fetch_b(qb0, f_b);
    advance_fetch();
    stage_a(0, ra);
    stage_b(0, rb);
    count_a(ra);
    count_b(rb);
    fetch_a(ra);
    const uint32_t* f_b_pending = f_b;                   // B's half of a fetch follows A's half a step later
    advance_fetch();
    if (write_thr) {
        // Clamped to the result range, which changes no output bit and keeps the folded terms exact.
        sh.thr[tid] = max(-K - 1, min(K + 1, thr_reg));
        if (tid < BN / 32) sh.flip[tid] = flip_reg;
    }
    stage_a(1, qa0);
    stage_b(1, qb0);
    count_a(qa0);
    count_b(qb0);
    __syncthreads();

    read_quads_a(0, 0, qa0);
    read_quads_b(0, 0, qb0);
    widen_step(qa0, qb0, 0, fa, fb);

    int buf = 0;                                         // LDS buffer of the K-tile being multiplied
    // K-steps 1 .. 7 of the K-tile in `buf` (step 0 has been issued; its successor's step 0 follows).
    // Memory operations of a K-tile, one per MFMA slot:
    //   step 0  global loads of B (stream position of the A loads issued in the step 7 before)
    //   1, 2    LDS reads of the second half's quads
    //   4, 5    the fetch registers (the K-tile two further on in the stream; past its end the last one again,
    //           written to a buffer that is not read any more) go to LDS and have their set bits counted: A, then B
    //   6       LDS reads of the next K-tile's first quads
    //   7       global loads of A for the following stream position
    auto steps_1_to_7 = [&]() {
        const int buf1 = buf == NBUF - 1 ? 0 : buf + 1;                  // next K-tile of the stream
        const int buf2 = buf1 == NBUF - 1 ? 0 : buf1 + 1;                // the one after it (written here)

        read_quads_a(buf, 1, qa1);
        k_step(qa0, qb0, 2, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x100, VALU);
        read_quads_b(buf, 1, qb1);
        k_step(qa0, qb0, 3, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x100, VALU);
        k_step(qa1, qb1, 0, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x100, VALU);

        // Every wavefront has finished the previous K-tile (whose buffer is written next) and has
        // written its part of the next one (written during the previous K-tile, read from step 6 of
        // this one on).
        __syncthreads();

        stage_a(buf2, ra);
        count_a(ra);
        k_step(qa1, qb1, 1, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x200, VALU + 1);
        stage_b(buf2, rb);
        count_b(rb);
        k_step(qa1, qb1, 2, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x200, VALU + 1);
        read_quads_a(buf1, 0, qa0);
        read_quads_b(buf1, 0, qb0);
        k_step(qa1, qb1, 3, std::false_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x100, VALU);
        fetch_a(ra);
        f_b_pending = f_b;
        k_step(qa0, qb0, 0, std::false_type{});
        // Keeps this step's widening here, between its MFMAs: its results are used after the
        // branches that follow, and would otherwise be computed there, with the matrix pipe idle.
#pragma unroll
        for (int i = 0; i < WM; ++i) asm volatile("" : "+v"(fa[i]));
#pragma unroll
        for (int j = 0; j < WN; ++j) asm volatile("" : "+v"(fb[j]));
        BNN_STEP_SCHEDULE(MFMAS, 0x020, VALU);
        buf = buf1;
        advance_fetch();
    };

    for (int tile_i = 0; tile_i < count; ++tile_i) {
        // Step 0 of the tile's first K-tile starts the sums.
        fetch_b(rb, f_b_pending);
        k_step(qa0, qb0, 1, std::true_type{});
        BNN_STEP_SCHEDULE(MFMAS, 0x020, VALU);
        for (int kt = 0; kt < n_ktiles - 1; ++kt) {
            steps_1_to_7();
            // The K-tile staged above was number kt + 2 of this output tile: with the last one the row sums are complete.
            if (__builtin_expect(kt + 2 == n_ktiles - 1, 0)) publish_row_sums();
            // Step 0 of the next K-tile.
            fetch_b(rb, f_b_pending);
            k_step(qa0, qb0, 1, std::false_type{});
            BNN_STEP_SCHEDULE(MFMAS, 0x020, VALU);
        }
        steps_1_to_7();

        // The row sums were published at least two barriers ago; the next tile's are published at least
        // one barrier (its first K-tile's) after this epilogue has read them.
        epilogue_bits<WM>(acc, sh, bn, min(first_row + BM * tile_i, last_row0), col0, wm, wn, fr, fh);
    }
}

}  // namespace big

// Workgroup b of the grid of tiles_n * strips.  The hardware places consecutive workgroups on the 8 dies
// (each with its own L2) in turn, so die d runs the workgroups b = d, d + 8, ...; they are given a compact
// block of die_strips strips times die_cols column tiles, chosen by the launcher so that the rows of A and
// B a die reads are as few as possible and its B tiles stay in its L2 over the strip's row tiles.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void xnor_gemm_mfma_big_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb, int K, int tiles_n,
    int strip_rows, int strip_extra, int die_strips, int die_cols, BnSignArgs bn) {
    using namespace big;
    __shared__ Shared sh;
    const int die = int(blockIdx.x) % 8, idx = int(blockIdx.x) / 8;     // idx < die_strips * die_cols
    const int dies_n = tiles_n / die_cols;
    const int strip = __builtin_amdgcn_readfirstlane((die / dies_n) * die_strips + idx / die_cols);
    const int col0 = __builtin_amdgcn_readfirstlane(((die % dies_n) * die_cols + idx % die_cols) * BN);
    // The column tile's thresholds and flip words, into registers: they go to LDS after the first operand
    // loads have been issued (run_row_tiles), so that no load of the kernel's start waits for another.
    const int thr_reg = bn.thr[col0 + threadIdx.x];
    uint32_t flip_reg = 0u;
    if (threadIdx.x < BN / 32) flip_reg = bn.flip_bits[(col0 >> 5) + threadIdx.x];
    // Rows [r_begin, r_end) of the strip (at least 256): strip_rows each, one more in the first strip_extra strips.
    const int r_begin = strip * strip_rows + min(strip, strip_extra);
    const int r_end = r_begin + strip_rows + (strip < strip_extra ? 1 : 0);
    const int rows = r_end - r_begin;
    const int rest = rows % BM_MAX;
    const int full = rows / BM_MAX + (rest > BM_MAX / 2 ? 1 : 0);      // 256-row tiles, the last one shifted up if partial
    const bool half = rest > 0 && rest <= BM_MAX / 2;                  // one 128-row tile at the strip's end

    run_row_tiles<4>(A, lda, B, ldb, K, bn, sh, r_begin, r_end - BM_MAX, full, col0, true, thr_reg, flip_reg);
    if (half) {
        __syncthreads();                                               // LDS buffers and row sums change hands
        run_row_tiles<2>(A, lda, B, ldb, K, bn, sh, r_end - BM_MAX / 2, r_end - BM_MAX / 2, 1, col0, false, 0, 0u);
    }
}

// Compute units of the current device (256 on MI355X), asked once.
static int big_compute_units() {
    static int n = 0;
    if (n == 0) {
        int dev = 0, cu = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0)
            return 256;
        n = cu;
    }
    return n;
}

// Row strips of the work split for an M x N product, 0 if the kernel does not take the shape: one workgroup
// per compute unit (a whole number of dies), N / 256 column tiles times `strips` row strips of at least 256 rows.
int64_t mfma_big_strips(int64_t M, int64_t N) {
    const int64_t slots = int64_t(big_compute_units()) / 8 * 8;
    if (N <= 0 || N % 256 != 0 || slots < 8) return 0;
    const int64_t tiles_n = N / 256;
    if (slots % tiles_n != 0) return 0;
    const int64_t strips = slots / tiles_n;
    return M / strips >= 256 ? strips : 0;
}

// Whether the work split suits the shape: a strip of one tile and a bit (257 .. 511 rows) pays two
// start-ups for little work and is left to the other kernels.
bool mfma_big_prefers(int64_t M, int64_t N) {
    const int64_t strips = mfma_big_strips(M, N);
    if (strips == 0) return false;
    const int64_t rows = M / strips;
    return rows >= 512 || (M % strips == 0 && rows == 256);
}

bool mfma_big_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                       int64_t K, const BnSignArgs& bn) {
    constexpr int64_t kTileK = 32 * kMfmaKT, kMaxLd = int64_t(1) << 22;
    if (K % kTileK != 0 || K < 4 * kTileK || K > kMfmaFoldMaxK || M > kMaxDim) return false;
    if (!aligned_to(A, 16) || !aligned_to(B, 16) || lda % 4 != 0 || ldb % 4 != 0 || lda >= kMaxLd || ldb >= kMaxLd)
        return false;
    if (!aligned_to(bn.out, 8) || bn.ld_out % 2 != 0) return false;       // 8-byte stores of word pairs
    return mfma_big_strips(M, N) > 0;
}

// BNN_ERR_UNSUPPORTED (nothing launched) unless the product is one this kernel takes.
int launch_xnor_gemm_mfma_big(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                              int64_t K, BnSignArgs bn, void* stream) {
    if (!mfma_big_supports(A, lda, B, ldb, M, N, K, bn)) return BNN_ERR_UNSUPPORTED;
    const int64_t strips = mfma_big_strips(M, N), tiles_n = N / 256, per_die = strips * tiles_n / 8;
    // A die's block of die_strips x die_cols workgroups: the rows of A and B it reads per K-tile, B counted
    // once per row tile of a strip if a die's B tiles do not fit in half of its 4 MB L2.
    const int64_t rows = ceil_div(M, strips), row_tiles = ceil_div(rows, 256);
    int64_t best_s = 0, best_cost = 0;
    for (int64_t ds = 1; ds <= strips && ds <= per_die; ++ds) {
        if (per_die % ds != 0 || strips % ds != 0) continue;
        const int64_t dc = per_die / ds;
        if (dc > tiles_n || tiles_n % dc != 0) continue;
        const bool b_resident = dc * 256 * (K / 8) <= (int64_t(2) << 20);
        const int64_t cost = ds * rows + dc * 256 * (b_resident ? 1 : row_tiles);
        if (best_s == 0 || cost < best_cost) {
            best_s = ds;
            best_cost = cost;
        }
    }
    if (best_s == 0) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(xnor_gemm_mfma_big_kernel, dim3(unsigned(strips * tiles_n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), A, lda, B, ldb, int(K), int(tiles_n), int(M / strips),
                       int(M % strips), int(best_s), int(per_die / best_s), bn);
    return check_launch();
}

}  // namespace bnn
