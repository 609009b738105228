// Bits-in, matrix-engine-inside binary product (Sec. 4 Eq. (5), the XnorDotProduct of Alg. 4) for
// short K: 96 < K <= 1152, the range of a first MLP layer on 28 x 28 inputs (K = 784) or of a 3 x 3
// convolution over 128 channels (K = 1152).
//
// With so few MFMA steps per output the kernel in xnor_gemm_mfma.hip spends most of a workgroup's
// life outside its K loop (first-tile load latency, epilogue, workgroup turnaround).  This one
// keeps the arithmetic (packed bits widened to fp4 in registers, v_mfma_f32_32x32x64_f8f6f4, row /
// column popcounts for the +-1 fix-up, the same epilogues) and changes the organisation:
//
//   - a workgroup owns one 128-column tile of B for its whole life: B's K bits (at most 144 bytes
//     per row) are staged in LDS once, with their popcounts, thresholds and flip words;
//   - it then walks over several 128-row tiles of A (every `groups`-th tile of the M direction).
//     The whole K extent of a tile sits in LDS at once, so a tile costs two barriers and its MFMA
//     steps run without any in between; the global loads of the next tile are in flight while the
//     current one is multiplied, and are written to LDS before the current tile's epilogue;
//   - only the K words that exist are multiplied: ceil(K / 128) * 2 steps of 64 bits, less the last one
//     where it would multiply nothing but zeros, instead of whole 512-bit K-tiles (13 instead of 16 steps
//     at K = 784).
//
// LDS layout of an operand tile: planes [quad q][half h] of 8-byte slots, slot r = row r's words
// 4q + 2h, 4q + 2h + 1.  Lane (row r = l % 32, half h = l / 32) of an MFMA operand reads slot r
// of plane (q, h): consecutive lanes, consecutive slots.  Step 2q + s multiplies word s of that
// pair, i.e. K words 4q + s (h = 0) and 4q + 2 + s (h = 1); the order of the K sum is free.
//
// Requirements (checked by the launcher): A, B 16-byte aligned, lda, ldb multiples of 4 words.
// The last quad of a row, where it is incomplete or holds pad bits, is loaded from the row's last
// four words (never past word K/32), moved into place and masked when it is written to LDS.
//
// Conv mode (CONV = true): A's rows are the receptive fields of a kh x kw convolution (Sec. 3.3)
// over a packed NHWC input with a multiple of 128 channels, gathered while the tile is fetched
// (implicit GEMM).  A quad is 4 channel words of one tap, so a staging thread's tap and channel
// offset are fixed for the kernel's life; the output pixel of its rows is stepped with carries
// from pass to pass and from tile to tile (no division inside the tile loop).  Taps outside the
// image are +1, i.e. all-ones words (zero padding through Eq. (1)), chosen at staging so that
// the loads stay unconditional (address clamped into the input).
#include <algorithm>
#include <type_traits>
#include <cstdint>

#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {

constexpr int kShortMaxQuads = 9;          // K <= 1152
constexpr int kShortMinWords = 4;          // K > 96: a row has at least one whole quad to load

// A 16-byte load from an address that is only 4-byte aligned (the last four words of a row).
__device__ inline uint4 load_quad_dword_aligned(const uint32_t* p) {
    uint4 v;
    __builtin_memcpy(&v, p, sizeof(v));
    return v;
}

template <int LANES>
__device__ inline int sum_over_lanes(int c) {
    static_assert(LANES == 8 || LANES == 16, "aligned groups of 8 or 16 lanes");
    c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);        // lane ^ 1
    c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);        // lane ^ 2
    c += __builtin_amdgcn_update_dpp(0, c, 0x141, 0xF, 0xF, true);       // row_half_mirror: 7 - lane within 8
    if (LANES == 16) c += __builtin_amdgcn_update_dpp(0, c, 0x140, 0xF, 0xF, true);   // row_mirror: 15 - lane
    return c;
}

// Words `first` .. `first + 3` of a quad that was loaded from the row's last four words
// (kw - 4 .. kw - 1): entries beyond the row read 0, the row's last word is masked.
__device__ inline uint4 align_last_quad(uint4 v, int shift, uint32_t tmask) {
    // shift = 4 - (valid words): the quad's word e is loaded word e + shift, and the row's last word is always
    // the last loaded one.  shift is the same for every thread: a branch, then one AND and register moves.
    const uint32_t last = v.w & tmask;
    switch (shift) {
        case 0: return make_uint4(v.x, v.y, v.z, last);
        case 1: return make_uint4(v.y, v.z, last, 0u);
        case 2: return make_uint4(v.z, last, 0u, 0u);
        default: return make_uint4(last, 0u, 0u, 0u);
    }
}

// Output pixel (image b, row y, column x) of a GEMM row, and a step of a fixed number of rows.
struct Pixel {
    int b, y, x;
};

__device__ inline Pixel pixel_of_row(int row, int Ho, int Wo) {
    const int t = row / Wo;
    return Pixel{t / Ho, t % Ho, row % Wo};
}

// p + d rows, d given as pixel_of_row(rows): one carry per coordinate.
__device__ inline void advance(Pixel& p, Pixel d, int Ho, int Wo) {
    p.x += d.x;
    if (p.x >= Wo) { p.x -= Wo; ++p.y; }
    p.y += d.y;
    if (p.y >= Ho) { p.y -= Ho; ++p.b; }
    p.b += d.b;
}

template <int TPR, bool FUSED, bool CONV>
__global__ __launch_bounds__(256, 3) void xnor_gemm_mfma_shortk_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, int groups,
    BnSignArgs bn, ConvArgs cv, uint32_t a_last_quad) {
    constexpr int WM = 2, WN = 2, BM = 64 * WM, BN = 64 * WN;
    static_assert(BM == BN, "one staging routine serves both operands");
    constexpr int PLANE = BM + 2;                       // 8-byte slots per plane (2 pad slots)
    constexpr int ROWS_PER_PASS = 256 / TPR;            // TPR threads fetch one row's quads
    constexpr int PASSES = BM / ROWS_PER_PASS;
    extern __shared__ uint2 lds_planes[];               // A planes, then B planes
    __shared__ __attribute__((aligned(16))) int pop_a[2][BM];
    __shared__ __attribute__((aligned(16))) float pop_af[2][FUSED ? BM : 4];
    __shared__ __attribute__((aligned(16))) int pop_b[BN];
    __shared__ __attribute__((aligned(16))) int thr_s[FUSED ? BN : 1];
    __shared__ uint32_t flip_s[FUSED ? BN / 32 : 1];
    __shared__ float colfix_s[FUSED ? BN : 1];          // column term of the folded threshold

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;
    const int kw = (K + 31) >> 5;
    const int kq = (kw + 3) >> 2;                       // quads per row
    const int n_fast = (K >> 5) >> 2;                   // quads of complete, unmasked words (kq or kq - 1)
    const uint32_t tmask = tail_mask(K);
    uint2* lds_a = lds_planes;
    uint2* lds_b = lds_planes + 2 * kq * PLANE;

    // Consecutive workgroup ids go round-robin to the 8 dies, each with its own L2.  A row of the packed
    // output is contiguous over the column tiles (16 bytes each), so the workgroups of one die take
    // neighbouring column tiles of the same rows: their partial lines meet in that die's L2.
    int n_tile = blockIdx.x % tiles_n, group = blockIdx.x / tiles_n;
    if (tiles_n % 8 == 0) {
        const int per_die = tiles_n / 8, die = blockIdx.x % 8, idx = blockIdx.x / 8;
        n_tile = die * per_die + idx % per_die;
        group = idx / per_die;
    }
    const int col0 = n_tile * BN;

    // Staging: thread (st_r, st_q) fetches quad st_q of rows st_r, st_r + ROWS_PER_PASS, ...
    const int st_q = tid % TPR, st_r = tid / TPR;
    const int word_off = st_q < n_fast ? 4 * st_q : kw - 4;       // always inside the row
    const int last_valid = kw - 4 * n_fast;                          // words of the last quad (when n_fast < kq)
    auto fetch = [&](const uint32_t* P, int64_t ld, int nrows, int r0, uint4 (&r)[PASSES]) __attribute__((always_inline)) {
#pragma unroll
        for (int l = 0; l < PASSES; ++l) {
            const int row = min(r0 + st_r + l * ROWS_PER_PASS, nrows - 1);   // rows beyond the matrix repeat its last row
            r[l] = load_quad_dword_aligned(P + int64_t(row) * ld + word_off);
        }
    };
    // conv: the tap (dy, dx relative to the output pixel's input position) and channel word of this
    // thread's quad, the output pixel of its first row of the next tile to fetch, and the steps.
    int tap_dy = 0, tap_dx = 0, tap_cw = 0;
    Pixel next_pix{0, 0, 0}, pass_step{0, 0, 0}, tile_step{0, 0, 0};
    uint32_t outside = 0u;                              // bit l: pass l's tap lies outside the image
    if (CONV) {
        const int tap = word_off / cv.Cw;
        tap_cw = word_off - tap * cv.Cw;
        tap_dy = tap / cv.kw - cv.pad;
        tap_dx = tap % cv.kw - cv.pad;
        next_pix = pixel_of_row(group * BM + st_r, cv.Ho, cv.Wo);
        pass_step = pixel_of_row(ROWS_PER_PASS, cv.Ho, cv.Wo);
        tile_step = pixel_of_row(groups * BM, cv.Ho, cv.Wo);
    }
    // Rows past the matrix (last tile only) step past the last image; their address is clamped to
    // the input's last quad, and what they compute is never stored.
    auto fetch_conv = [&](uint4 (&r)[PASSES]) __attribute__((always_inline)) {
        Pixel p = next_pix;
        outside = 0u;
#pragma unroll
        for (int l = 0; l < PASSES; ++l) {
            const int y = p.y * cv.stride + tap_dy, x = p.x * cv.stride + tap_dx;
            const bool inside = y >= 0 && y < cv.H && x >= 0 && x < cv.W;
            const int yc = min(max(y, 0), cv.H - 1), xc = min(max(x, 0), cv.W - 1);
            const uint32_t off = (uint32_t(p.b * cv.H + yc) * uint32_t(cv.W) + uint32_t(xc)) * uint32_t(cv.Cw) + uint32_t(tap_cw);
            r[l] = *reinterpret_cast<const uint4*>(A + min(off, a_last_quad));
            outside |= inside ? 0u : 1u << l;
            advance(p, pass_step, cv.Ho, cv.Wo);
        }
        advance(next_pix, tile_step, cv.Ho, cv.Wo);
    };
    auto fetch_a = [&](int tile, uint4 (&r)[PASSES]) __attribute__((always_inline)) {
        if (CONV) fetch_conv(r);
        else fetch(A, lda, M, tile * BM, r);
    };
    // Writes the fetched quads to their two planes and returns nothing; cnt[l] = set bits written.
    auto stage = [&](uint2* planes, const uint4 (&r)[PASSES], int (&cnt)[PASSES], uint32_t ones) __attribute__((always_inline)) {
#pragma unroll
        for (int l = 0; l < PASSES; ++l) {
            uint4 v = r[l];
            if (st_q >= n_fast) v = align_last_quad(v, 4 - last_valid, tmask);
            if (CONV && ((ones >> l) & 1u)) v = make_uint4(~0u, ~0u, ~0u, ~0u);
            cnt[l] = 0;
            if (st_q < kq) {
                const int row = st_r + l * ROWS_PER_PASS;
                planes[(2 * st_q) * PLANE + row] = make_uint2(v.x, v.y);
                planes[(2 * st_q + 1) * PLANE + row] = make_uint2(v.z, v.w);
                cnt[l] = popc4(v);
            }
        }
    };

    uint4 ra[PASSES];
    int cnt[PASSES];
    {
        // B tile, once: bits, column popcounts, thresholds and flip words.
        uint4 rb[PASSES];
        fetch(B, ldb, N, col0, rb);
        if (FUSED) {
            // No result exceeds K in magnitude, so clamping a threshold to [-K-1, K+1] changes no
            // output bit and keeps the bounds the epilogue derives from it inside int32.
            if (tid < BN) thr_s[tid] = col0 + tid < N ? max(-K - 1, min(K + 1, bn.thr[col0 + tid])) : 0;
            if (tid < BN / 32) flip_s[tid] = col0 + 32 * tid < N ? bn.flip_bits[(col0 >> 5) + tid] : 0u;
        }
        if (group < tiles_m) fetch_a(group, ra);
        stage(lds_b, rb, cnt, 0u);
#pragma unroll
        for (int l = 0; l < PASSES; ++l) {
            const int c = sum_over_lanes<TPR>(cnt[l]);
            if (st_q == 0) pop_b[st_r + l * ROWS_PER_PASS] = 2 * c;
        }
    }
    auto stage_a = [&](int buf) __attribute__((always_inline)) {
        stage(lds_a, ra, cnt, outside);
#pragma unroll
        for (int l = 0; l < PASSES; ++l) {
            const int c = sum_over_lanes<TPR>(cnt[l]);
            if (st_q == 0) {
                pop_a[buf][st_r + l * ROWS_PER_PASS] = 2 * c;
                if (FUSED) pop_af[buf][st_r + l * ROWS_PER_PASS] = 0.5f * float(c);
            }
        }
    };
    if (group < tiles_m) stage_a(0);
    __syncthreads();
    // Read by the first epilogue, which follows another barrier.
    if (FUSED && tid < BN) colfix_s[tid] = fold_column_term(thr_s[tid], K, pop_b[tid]);

    // Operand slots of this lane: plane (q, fh), rows wm*64 + 32*i + fr (A) / wn*64 + 32*j + fr (B).
    const uint2* rd_a = lds_a + fh * PLANE + wm * 32 * WM + fr;
    const uint2* rd_b = lds_b + fh * PLANE + wn * 32 * WN + fr;

    // Steps of 64 bits: two per quad, except that a last quad holding a single word (K words = 4q + 1) has
    // nothing but zeros in its second step (words 4q + 1 and 4q + 3), which is then left out.
    const int n_steps = 2 * kq - ((((K + 31) >> 5) & 3) == 1 ? 1 : 0);
    int buf = 0;
    for (int tile_m = group; tile_m < tiles_m; tile_m += groups, buf ^= 1) {
        const bool more = tile_m + groups < tiles_m;
        if (more) fetch_a(tile_m + groups, ra);                      // in flight during the MFMA steps

        v16f acc[WM][WN];
        if constexpr (!FUSED) {                     // (the int32 form has no registers to spare for the peeled first step)
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        }
        uint2 a_cur[WM], b_cur[WN];
#pragma unroll
        for (int i = 0; i < WM; ++i) a_cur[i] = rd_a[i * 32];
#pragma unroll
        for (int j = 0; j < WN; ++j) b_cur[j] = rd_b[j * 32];
        // One step of 64 bits on word s of the current pairs.  first: the tile's first step, which in the fused
        // form starts the sums with a zero addend instead of cleared accumulators.
        auto step = [&](int s, auto first_tag) {
            constexpr bool FIRST = FUSED && decltype(first_tag)::value;
            v8i fa[WM], fb[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) fa[i] = widen_fp4_a(s == 0 ? a_cur[i].x : a_cur[i].y);
#pragma unroll
            for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(s == 0 ? b_cur[j].x : b_cur[j].y);
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    v16f addend = acc[i][j];
                    if (FIRST) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) addend[v] = 0.0f;
                    }
                    // fused: operands swapped, the accumulators hold the transposed blocks (mfma_epilogue_bits)
                    if (FUSED)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[j], fa[i], addend, 4 /* fp4 */,
                                                                                    4 /* fp4 */, 0, 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fa[i], fb[j], addend, 4 /* A: fp4 */,
                                                                                    4 /* B: fp4 */, 0, 0, 0, 0);
                }
        };
        // A quad is two steps (n_steps says whether the last quad's second one exists); the pairs of the next
        // quad are read during the current one (the last quad re-reads its own: no branch around the reads).
        auto quad = [&](int q, auto first_tag) {
            const int qn = min(q + 1, kq - 1);
            uint2 a_nxt[WM], b_nxt[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) a_nxt[i] = rd_a[2 * qn * PLANE + i * 32];
#pragma unroll
            for (int j = 0; j < WN; ++j) b_nxt[j] = rd_b[2 * qn * PLANE + j * 32];
            step(0, first_tag);
            if (2 * q + 1 < n_steps) step(1, std::false_type{});
#pragma unroll
            for (int i = 0; i < WM; ++i) a_cur[i] = a_nxt[i];
#pragma unroll
            for (int j = 0; j < WN; ++j) b_cur[j] = b_nxt[j];
        };
        if constexpr (FUSED) {
            quad(0, std::true_type{});
            for (int q = 1; q < kq; ++q) quad(q, std::false_type{});
        } else {
            for (int q = 0; q < kq; ++q) quad(q, std::false_type{});
        }

        __syncthreads();                            // every wavefront has read this tile's planes
        if (more) stage_a(buf ^ 1);                 // next tile's bits and row sums (the other pop_a half)
        if constexpr (FUSED)
            mfma_epilogue_bits<WM, WN>(acc, pop_a[buf], pop_af[buf], pop_b, thr_s, flip_s, colfix_s, bn, M, N, K,
                                       tile_m * BM, col0, wm, wn, fr, fh);
        else
            mfma_epilogue<WM, WN, false, false>(acc, pop_a[buf], pop_af[buf], pop_b, thr_s, flip_s, C, ldc, bn, M, N, K,
                                                tile_m * BM, col0, wm, wn, fr, fh);
        __syncthreads();                            // next tile staged; this tile's row sums no longer needed
    }
}

bool mfma_shortk_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t K) {
    const int64_t kw = ceil_div(K, 32);
    return kw >= kShortMinWords && kw <= 4 * kShortMaxQuads && aligned_to(A, 16) && aligned_to(B, 16) &&
           lda % 4 == 0 && ldb % 4 == 0;
}

// Workgroups per 128-column tile: every workgroup of a column tile takes every `groups`-th row tile.
// Measured on MI355X (10000 x 4096 x 784, 262144 x 128 x 1152): what counts is that three workgroups
// are resident on every compute unit from start to end, so that one's loads, barriers and epilogue
// overlap the others' MFMA steps; an even split of the row tiles matters less.  So: as many
// workgroups as the chip holds at once (3 x 256), at most one per row tile.
static int shortk_groups(int64_t tiles_m, int64_t tiles_n) {
    constexpr int64_t kSlots = 3 * 256;
    return int(std::max<int64_t>(1, std::min<int64_t>(tiles_m, kSlots / tiles_n)));
}

template <bool FUSED, bool CONV>
static int launch_shortk(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc,
                         int64_t M, int64_t N, int64_t K, BnSignArgs bn, ConvArgs cv, void* stream) {
    const int64_t tiles_m = ceil_div(M, 128), tiles_n = ceil_div(N, 128);
    const int groups = shortk_groups(tiles_m, tiles_n);
    if (tiles_n * groups > kMaxDim) return BNN_ERR_UNSUPPORTED;
    const int64_t kq = ceil_div(ceil_div(K, 32), 4);
    const size_t lds_bytes = size_t(2) * 2 * kq * (128 + 2) * sizeof(uint2);
    // conv: word offset of the input's last 16-byte quad (the input holds whole images of M / (Ho * Wo)).
    const uint32_t a_last_quad =
        CONV ? uint32_t(M / (int64_t(cv.Ho) * cv.Wo) * cv.H * cv.W * cv.Cw - 4) : 0u;
    const dim3 grid(unsigned(tiles_n * groups));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (kq <= 8)
        hipLaunchKernelGGL((xnor_gemm_mfma_shortk_kernel<8, FUSED, CONV>), grid, dim3(256), lds_bytes, s, A, lda, B, ldb,
                           C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), groups, bn, cv, a_last_quad);
    else
        hipLaunchKernelGGL((xnor_gemm_mfma_shortk_kernel<16, FUSED, CONV>), grid, dim3(256), lds_bytes, s, A, lda, B, ldb,
                           C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), groups, bn, cv, a_last_quad);
    return check_launch();
}

int launch_xnor_gemm_mfma_shortk(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                 int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    if (!mfma_shortk_supports(A, lda, B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    return launch_shortk<false, false>(A, lda, B, ldb, C, ldc, M, N, K, BnSignArgs{}, ConvArgs{}, stream);
}

int launch_xnor_gemm_mfma_shortk_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                       int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    if (!mfma_shortk_supports(A, lda, B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    return launch_shortk<true, false>(A, lda, B, ldb, nullptr, 0, M, N, K, bn, ConvArgs{}, stream);
}

// Conv mode: `in` is the packed NHWC input (16-byte aligned, a multiple of 128 channels: checked by
// the caller), B the packed filters [N][kh*kw*Cw].  K = kh*kw*Cin is then a multiple of 128.
bool conv_shortk_supports(const uint32_t* B, int64_t ldb, int64_t K) {
    return K <= 128 * kShortMaxQuads && aligned_to(B, 16) && ldb % 4 == 0;
}

int launch_conv_mfma_shortk(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                            int64_t N, int64_t K, ConvArgs cv, void* stream) {
    if (!conv_shortk_supports(B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    return launch_shortk<false, true>(in, 0, B, ldb, C, ldc, M, N, K, BnSignArgs{}, cv, stream);
}

int launch_conv_mfma_shortk_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                                  int64_t K, BnSignArgs bn, ConvArgs cv, void* stream) {
    if (!conv_shortk_supports(B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    return launch_shortk<true, true>(in, 0, B, ldb, nullptr, 0, M, N, K, bn, cv, stream);
}

}  // namespace bnn
