// Whole-tile form of the bits-in, matrix-engine-inside kernel for the large products of Alg. 4
// (a_k = XnorDotProduct(a^b_{k-1}, W^b_k), Sec. 4 Eq. (5); with FUSED also a^b_k = Sign(BatchNorm(a_k))).
//
// Arithmetic, operand widening, LDS layout and epilogues are those of xnor_gemm_mfma.hip (256 x 128
// tiles, 2 x 2 wavefronts of 4 x 2 accumulator blocks).  It takes only products where nothing has to be
// checked per element (the launcher refuses the rest, which stay with xnor_gemm_mfma.hip):
//   - K a multiple of 512 (whole K-tiles: no masking, no partial loads), 1024 <= K <= 2^24;
//   - N a multiple of 128 (whole column tiles), M >= 256; the last row tile is SHIFTED up to end at
//     row M instead of being padded, so every tile row exists (rows shared with the previous tile
//     are computed twice and written twice with the same values);
//   - operands that allow 16-byte loads, leading dimensions below 2^22 words.
// With whole tiles every global address is `wavefront-uniform tile address + constant 32-bit lane offset`:
// the per-lane 64-bit row pointers of the general kernel (12 registers, recomputed per tile) and the
// 64-bit address per int32 store are gone.  The int32 epilogue is where that shows: 128 stores per
// lane at scalar bases (8192^3 199 -> 190 us with one workgroup per tile).
//
// A workgroup walks over the output tiles blockIdx.x, blockIdx.x + gridDim.x, ... (the stride is kept a
// multiple of the number of dies, so a workgroup's tiles keep to one die's L2 panel); during the last
// K-tile of an output tile the first K-tile of the next one is fetched, and it is staged before the
// epilogue runs.  Two launch shapes:
//   - one workgroup per tile (grid = tiles, no walk): the hardware hands tiles to whichever slot frees
//     up first, which balances a long run of tiles better than any fixed assignment (32768 x 4096 x 4096
//     int32: 209 us vs 214 us walked);
//   - one workgroup per resident slot (two per compute unit) walking over the tiles: the better form when
//     the last round of tiles is partial, because every compute unit then gets the same share of it
//     (10000 x 4096 x 4096 fused: 57.5 -> 55.5 us; 9216 x 4096 x 2048 int32: 41.3 -> 39.1 us).
#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {

// 16-byte load at a wavefront-uniform address plus a per-lane 32-bit byte offset.
__device__ inline uint4 load16_at(const uint32_t* uniform_base, uint32_t lane_byte_offset) {
    return *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(uniform_base) + lane_byte_offset);
}

// One 4-byte vector store at `uniform row address + per-lane byte offset (+ 128 * J)`: the scalar-base form
// of global_store_dword, spelled out because the compiler otherwise forms (and keeps, and spills) a 64-bit
// address per lane and element.  Cache policy of the store: THROUGH = agent scope (sc1: written through the
// die's L2), else non-temporal.  Measured on whole int32 products (8192^3: 189.5 vs 194.0 us; 8192 x 8192 x 2048:
// 70.4 vs 80.4 us; 8192 x 4096 x 8192: 97.1 vs 101.6 us; from about 330 MB of output on the two are level, one
// shape of 537 MB 3 % slower written through): the launcher writes through up to kThroughMaxBytes of output.
template <int J, bool THROUGH>
__device__ inline void store_at(int32_t* uniform_row, uint32_t lane_byte_offset, int value) {
    static_assert(J == 0 || J == 1, "column block of the wavefront");
    if (J == 0 && THROUGH)
        asm volatile("global_store_dword %0, %1, %2 sc1" : : "v"(lane_byte_offset), "v"(value), "s"(uniform_row) : "memory");
    else if (J == 0)
        asm volatile("global_store_dword %0, %1, %2 nt" : : "v"(lane_byte_offset), "v"(value), "s"(uniform_row) : "memory");
    else if (THROUGH)
        asm volatile("global_store_dword %0, %1, %2 offset:128 sc1"
                     : : "v"(lane_byte_offset), "v"(value), "s"(uniform_row) : "memory");
    else
        asm volatile("global_store_dword %0, %1, %2 offset:128 nt"
                     : : "v"(lane_byte_offset), "v"(value), "s"(uniform_row) : "memory");
}
constexpr int64_t kThroughMaxBytes = int64_t(320) << 20;

// int32 epilogue for tiles that lie wholly inside the matrix: dot = K - 2pa - 2pb + 4S for the
// wavefront's 4 x 2 accumulator blocks (register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column
// l%32 of its 32 x 32 block).  Every store address is a wavefront-uniform row address (scalar
// registers) plus one per-lane 32-bit offset; the wavefront's second column block is 128 bytes
// further on.  wm / wn / row0 / col0 must be wavefront-uniform.  pop_a / pop_b hold 2 * popcount
// per tile row / column.
template <int WM, int WN, bool THROUGH>
__device__ inline void persist_epilogue_int32(const v16f (&acc)[WM][WN], const int* pop_a, const int* pop_b,
                                              int32_t* __restrict__ C, int64_t ldc, int K, int row0, int col0, int wm,
                                              int wn, int fr, int fh) {
    static_assert(WN == 2, "two column blocks of 32 int32 = 128 bytes apart");
    const uint32_t lane_off = (uint32_t(4 * fh) * uint32_t(ldc) + uint32_t(fr)) * 4u;      // ldc < 2^27
    int base_n[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) base_n[j] = K - pop_b[wn * 32 * WN + j * 32 + fr];
    int32_t* tile_base = C + (int64_t(row0 + wm * 32 * WM) * ldc + col0 + wn * 32 * WN);   // uniform
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
            const int ml = i * 32 + 8 * vq;                                  // row of the wavefront's 128, uniform part
            const int4 pa2 = *reinterpret_cast<const int4*>(&pop_a[wm * 32 * WM + ml + 4 * fh]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int pa = e == 0 ? pa2.x : e == 1 ? pa2.y : e == 2 ? pa2.z : pa2.w;
                int32_t* row = tile_base + int64_t(ml + e) * ldc;
                store_at<0, THROUGH>(row, lane_off, base_n[0] - pa + (int(acc[i][0][4 * vq + e]) << 2));
                store_at<1, THROUGH>(row, lane_off, base_n[1] - pa + (int(acc[i][1][4 * vq + e]) << 2));
            }
        }
}

template <bool FUSED, bool THROUGH>
__global__ __launch_bounds__(256, 2) void xnor_gemm_mfma_persist_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn) {
    constexpr int WM = 4, WN = 2;
    constexpr int BM = 64 * WM, BN = 64 * WN;          // 2 x 2 wavefronts
    constexpr int PLANE_A = BM + 2, PLANE_B = BN + 2;  // 16-byte slots per quad plane (2 pad slots)
    constexpr int ST_ROWS = 256 / kMfmaKQ;             // rows covered by one staging pass
    constexpr int LOADS_A = BM / ST_ROWS, LOADS_B = BN / ST_ROWS;
    static_assert(kMfmaKQ == 4, "the row-popcount reduction below assumes 4 staging lanes per row");
    __shared__ uint4 lds_a[2][kMfmaKQ * PLANE_A];
    __shared__ uint4 lds_b[2][kMfmaKQ * PLANE_B];
    __shared__ __attribute__((aligned(16))) int pop_a[BM];
    __shared__ __attribute__((aligned(16))) int pop_b[BN];
    __shared__ __attribute__((aligned(16))) float pop_af[FUSED ? BM : 4];
    __shared__ __attribute__((aligned(16))) int thr_s[FUSED ? BN : 1];
    __shared__ uint32_t flip_s[FUSED ? BN / 32 : 1];
    __shared__ float colfix_s[FUSED ? BN : 1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // a scalar: uniform per wavefront
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;
    const int n_ktiles = K / (32 * kMfmaKT);            // whole K-tiles only
    const int st_q = tid % kMfmaKQ, st_r = tid / kMfmaKQ;
    // Byte offset of this thread's quad inside a staging pass of 64 rows (leading dimensions < 2^22 words).
    const uint32_t a_off = (uint32_t(st_r) * uint32_t(lda) + 4u * st_q) * 4u;
    const uint32_t b_off = (uint32_t(st_r) * uint32_t(ldb) + 4u * st_q) * 4u;

    const int total_tiles = tiles_m * tiles_n;
    int tile = blockIdx.x;
    int tile_m, tile_n;
    tile_of_block(tile, tiles_m, tiles_n, tile_m, tile_n);
    // (row0, col0) of the tile whose K-tiles are being fetched.  The tile order divides by run-time
    // values on the vector ALU; readfirstlane brings the (uniform) result back into scalar registers so
    // that tile addresses are scalar bases.
    int row0 = __builtin_amdgcn_readfirstlane(min(tile_m * BM, M - BM));
    int col0 = __builtin_amdgcn_readfirstlane(tile_n * BN);

    uint4 ra[LOADS_A], rb[LOADS_B];
    int cnt_a[LOADS_A], cnt_b[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) cnt_a[l] = 0;
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) cnt_b[l] = 0;

    auto fetch = [&](int kt) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l)
            ra[l] = load16_at(A + (int64_t(row0 + l * ST_ROWS) * lda + kt * kMfmaKT), a_off);
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l)
            rb[l] = load16_at(B + (int64_t(col0 + l * ST_ROWS) * ldb + kt * kMfmaKT), b_off);
    };
    // Writes the fetched words to LDS and adds their set bits to this thread's row sums.
    auto stage = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            cnt_a[l] += popc4(ra[l]);
            lds_a[buf][st_q * PLANE_A + st_r + l * ST_ROWS] = ra[l];
        }
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            cnt_b[l] += popc4(rb[l]);
            lds_b[buf][st_q * PLANE_B + st_r + l * ST_ROWS] = rb[l];
        }
    };
    // The tile's thresholds (clamped to the result range, which changes no output bit and keeps the
    // epilogue's bounds inside int32 for any caller-given value) and flip words, into LDS.
    auto load_thresholds = [&]() {
        if (tid < BN) thr_s[tid] = max(-K - 1, min(K + 1, bn.thr[col0 + tid]));
        if (tid < BN / 32) flip_s[tid] = bn.flip_bits[(col0 >> 5) + tid];
    };
    // Row sums of the finished tile: the 4 threads that staged the quads of one row are neighbouring
    // lanes.  pop_a / pop_b hold 2 * popcount.
    auto publish_row_sums = [&]() {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            int c = cnt_a[l];
            c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);       // lane ^ 1
            c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);       // lane ^ 2
            if (st_q == 0) {
                pop_a[st_r + l * ST_ROWS] = 2 * c;
                if (FUSED) pop_af[st_r + l * ST_ROWS] = 0.5f * float(c);
            }
            cnt_a[l] = 0;
        }
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            int c = cnt_b[l];
            c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);
            c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);
            if (st_q == 0) {
                pop_b[st_r + l * ST_ROWS] = 2 * c;
                if (FUSED) colfix_s[st_r + l * ST_ROWS] = fold_column_term(thr_s[st_r + l * ST_ROWS], K, 2 * c);
            }
            cnt_b[l] = 0;
        }
    };

    v16f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (FUSED) load_thresholds();
    fetch(0);
    stage(0);
    __syncthreads();

    int buf = 0;                                        // LDS buffer of the K-tile being multiplied
    bool more = true;
    while (more) {
        const int out_row0 = row0, out_col0 = col0;     // row0 / col0 move on to the next tile before this one's epilogue
        const bool has_next = tile + int(gridDim.x) < total_tiles;
        for (int kt = 0; kt < n_ktiles; ++kt) {
            const bool last = kt + 1 == n_ktiles;
            if (!last) {
                fetch(kt + 1);
            } else if (has_next) {
                tile_of_block(tile + int(gridDim.x), tiles_m, tiles_n, tile_m, tile_n);
                row0 = __builtin_amdgcn_readfirstlane(min(tile_m * BM, M - BM));
                col0 = __builtin_amdgcn_readfirstlane(tile_n * BN);
                fetch(0);
            }

            // The lane's 8 words are quads 2*fh and 2*fh+1 of its tile row; each quad feeds 4 steps.
#pragma unroll
            for (int hq = 0; hq < 2; ++hq) {
                uint4 aw[WM], bw[WN];
#pragma unroll
                for (int i = 0; i < WM; ++i) aw[i] = lds_a[buf][(2 * fh + hq) * PLANE_A + wm * 32 * WM + i * 32 + fr];
#pragma unroll
                for (int j = 0; j < WN; ++j) bw[j] = lds_b[buf][(2 * fh + hq) * PLANE_B + wn * 32 * WN + j * 32 + fr];
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    v8i fa[WM], fb[WN];
#pragma unroll
                    for (int i = 0; i < WM; ++i) fa[i] = widen_fp4_a(quad_word(aw[i], s));
#pragma unroll
                    for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(quad_word(bw[j], s));
                    // Unit block scales: literal zero scale operands select the plain
                    // v_mfma_f32_32x32x64_f8f6f4.  The fused form multiplies with the operands
                    // swapped, so its accumulator blocks are the transposes of the output blocks
                    // and the epilogue can pack a row's bits inside a lane.
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int j = 0; j < WN; ++j) {
                            if (FUSED)
                                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                    fb[j], fa[i], acc[i][j], 4 /* fp4 */, 4 /* fp4 */, 0, 0, 0, 0);
                            else
                                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                    fa[i], fb[j], acc[i][j], 4 /* fp4 */, 4 /* fp4 */, 0, 0, 0, 0);
                        }
                }
            }

            // Ordering pin: keeps the staging of the fetched tile (and with it the wait for the
            // global loads issued at the top of this iteration) behind the MFMA steps.
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) asm volatile("" : "+v"(acc[i][j]) : : "memory");

            if (!last) {
                stage(buf ^ 1);
            } else {
                // The finished tile's row sums go out before the next tile's first K-tile is counted.
                publish_row_sums();
                if (has_next) stage(buf ^ 1);
            }
            __syncthreads();
            buf ^= 1;
        }

        if constexpr (FUSED)
            mfma_epilogue_bits<WM, WN>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, colfix_s, bn, M, N, K, out_row0,
                                       out_col0, wm, wn, fr, fh);
        else
            persist_epilogue_int32<WM, WN, THROUGH>(acc, pop_a, pop_b, C, ldc, K, out_row0, out_col0, wm, wn, fr, fh);
        more = has_next;
        if (more) {
            // The next tile's first K-tile is already staged.  The epilogue has read the row sums and
            // the thresholds from LDS; the barrier keeps the new thresholds (and, K-tiles later, the
            // new row sums) from overtaking those reads.  The thresholds are read again when the row
            // sums are published, at least one barrier from here (n_ktiles >= 2).
            tile += int(gridDim.x);
            __syncthreads();
            if (FUSED) load_thresholds();
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        }
    }
}

// Compute units of the current device (256 on MI355X), asked once.
static int compute_units() {
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

// Resident workgroup slots of the persistent kernel: two per compute unit, a whole number of dies.
int64_t mfma_persist_slots() { return int64_t(2) * compute_units() / 8 * 8; }

// Whether the product is one this kernel takes (ldc: of the int32 output, ignored when fused); walk: as a
// tile walk of one workgroup per resident slot, which needs more tiles than slots.
bool mfma_persist_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t ldc, int64_t M,
                           int64_t N, int64_t K, bool fused, bool walk) {
    constexpr int64_t kTileM = 256, kTileN = 128, kTileK = 32 * kMfmaKT, kMaxLd = int64_t(1) << 22;
    if (K % kTileK != 0 || K < 2 * kTileK || K > kMfmaMaxAcc || N % kTileN != 0 || M < kTileM) return false;
    if (!aligned_to(A, 16) || !aligned_to(B, 16) || lda % 4 != 0 || ldb % 4 != 0 || lda >= kMaxLd || ldb >= kMaxLd)
        return false;
    if (!fused && ldc >= (int64_t(1) << 27)) return false;       // 32-bit lane byte offsets (16 * ldc + 124) in the int32 epilogue
    const int64_t tiles = ceil_div(M, kTileM) * (N / kTileN);
    const int64_t slots = mfma_persist_slots();
    return tiles <= kMaxDim && (!walk || (slots >= 8 && tiles > slots));
}

// BNN_ERR_UNSUPPORTED (nothing launched) unless the product is one this kernel takes.
// fused: bn holds thresholds, flip words and the output.  walk: one workgroup per resident slot walking
// over the tiles, else one workgroup per tile.
int launch_xnor_gemm_mfma_persist(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                  int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, bool walk, BnSignArgs bn,
                                  void* stream) {
    if (!mfma_persist_supports(A, lda, B, ldb, ldc, M, N, K, fused, walk)) return BNN_ERR_UNSUPPORTED;
    const int64_t tiles_m = ceil_div(M, 256), tiles_n = N / 128;
    const int64_t slots = walk ? mfma_persist_slots() : tiles_m * tiles_n;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fused)
        hipLaunchKernelGGL((xnor_gemm_mfma_persist_kernel<true, false>), dim3(unsigned(slots)), dim3(256), 0, s, A, lda, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn);
    else if (M * N * int64_t(sizeof(int32_t)) <= kThroughMaxBytes)
        hipLaunchKernelGGL((xnor_gemm_mfma_persist_kernel<false, true>), dim3(unsigned(slots)), dim3(256), 0, s, A, lda, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn);
    else
        hipLaunchKernelGGL((xnor_gemm_mfma_persist_kernel<false, false>), dim3(unsigned(slots)), dim3(256), 0, s, A, lda, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn);
    return check_launch();
}

}  // namespace bnn
