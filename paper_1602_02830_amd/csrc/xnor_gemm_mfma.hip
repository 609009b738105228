// Bits-in, matrix-engine-inside variant of the binary product of Sec. 4 / Alg. 4.
//
// Operands stay packed 32 per word in HBM and LDS (the 32x smaller footprint
// the paper argues for); only inside registers is each bit widened to a 4-bit
// float (E2M1: code 0b0010 = 1.0, 0b0000 = 0.0) and fed to
// v_mfma_scale_f32_32x32x64_f8f6f4, whose fp32 accumulation of 0/1 products is
// exact for K < 2^24.  With a, b in {0,1} standing for -1/+1:
//
//   sum_k (2a-1)(2b-1) = K - 2*popcount(A_m) - 2*popcount(B_n) + 4 * sum_k a*b
//
// so the +-1 product of Eq. (5) is the matrix-engine sum S plus per-row and
// per-column popcounts, which the staging threads gather for free while they
// copy the tile.  Pad bits and rows outside the matrix are zeroed at staging
// and therefore contribute to neither S nor the popcounts.
//
// Widening: element k of a word lands in operand register k%4, nibble k/4, for
// both operands (the sum over k does not depend on its order).  The E2M1 codes
// 0b0001, 0b0010, 0b0100 are 0.5, 1.0, 2.0, so most registers are a bare mask of
// the word and only the product of the two sides has to be 1:
//   register   0               1             2               3
//   A side     w & 0x1111.. (0.5)  w & 0x2222.. (1)  w & 0x4444.. (2)  (w>>2) & 0x2222.. (1)
//   B side     (w<<2) & 0x4444.. (2)  w & 0x2222.. (1)  (w>>2) & 0x1111.. (0.5)  (w>>2) & 0x2222.. (1)
// i.e. 5 vector-ALU operations per 32 elements on the A side, 6 on the B side.
//
// Workgroup = 256 threads = 2 x 2 wavefronts; a wavefront owns WM x WN blocks
// of 32 x 32 outputs (fp32 accumulators).  K advances 16 words (512 bits) per
// staged tile = 8 MFMA steps of 64 bits: lane (row r = l%32, half h = l/32) of
// a fragment owns words [8h, 8h+8) of its row, read with two ds_read_b128.
// The tile is long enough that the global loads of the next tile, issued
// before the MFMA steps, have landed when they are staged.
#include "bnn_internal.h"
#include "gemm_staging.h"

namespace bnn {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMfmaKT = 16;         // words of K per staged tile
constexpr int kMfmaKQ = kMfmaKT / 4;  // 16-byte quads per row per tile
constexpr int kMfmaSteps = kMfmaKT / 2;  // MFMA steps per tile (each consumes one word from each lane half)
constexpr int64_t kMfmaMaxK = int64_t(1) << 24;   // exact fp32 accumulation of 0/1 products

__device__ inline v8i widen_fp4_a(uint32_t w) {
    v8i f = {int(w & 0x11111111u), int(w & 0x22222222u), int(w & 0x44444444u), int((w >> 2) & 0x22222222u),
             0, 0, 0, 0};
    return f;
}

__device__ inline v8i widen_fp4_b(uint32_t w) {
    const uint32_t r = w >> 2;
    v8i f = {int((w << 2) & 0x44444444u), int(w & 0x22222222u), int(r & 0x11111111u), int(r & 0x22222222u),
             0, 0, 0, 0};
    return f;
}

__device__ inline int popc4(uint4 v) { return __popc(v.x) + __popc(v.y) + __popc(v.z) + __popc(v.w); }

template <int WM, int WN, bool VEC, bool FUSED>
__global__ __launch_bounds__(256, 2) void xnor_gemm_mfma_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn) {
    constexpr int BM = 64 * WM, BN = 64 * WN;          // 2 x 2 wavefronts
    constexpr int PLANE_A = BM + 2, PLANE_B = BN + 2;  // 16-byte slots per quad plane (2 pad slots)
    constexpr int ST_ROWS = 256 / kMfmaKQ;             // rows covered by one staging pass
    constexpr int LOADS_A = BM / ST_ROWS, LOADS_B = BN / ST_ROWS;
    static_assert(BM % ST_ROWS == 0 && BN % ST_ROWS == 0, "tile rows must divide among the staging threads");
    static_assert(kMfmaKQ == 4, "the row-popcount reduction below assumes 4 staging lanes per row");
    __shared__ uint4 lds_a[2][kMfmaKQ * PLANE_A];
    __shared__ uint4 lds_b[2][kMfmaKQ * PLANE_B];
    __shared__ __attribute__((aligned(16))) int pop_a[BM];
    __shared__ __attribute__((aligned(16))) int pop_b[BN];

    int tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;
    const int kw = (K + 31) >> 5;
    const uint32_t tmask = tail_mask(K);
    const int n_ktiles = (kw + kMfmaKT - 1) / kMfmaKT;

    const int st_q = tid % kMfmaKQ, st_r = tid / kMfmaKQ;
    // Complete K-tiles take branch-free loads (row clamped into the matrix, zeroed at staging
    // if it does not exist); the last, partial K-tile goes through the checked, masking loader.
    const int n_full_ktiles = (K >> 5) / kMfmaKT;
    const uint32_t* pa[LOADS_A];
    const uint32_t* pb[LOADS_B];
    bool live_a[LOADS_A], live_b[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) {
        const int r = row0 + st_r + l * ST_ROWS;
        live_a[l] = r < M;
        pa[l] = A + int64_t(min(r, M - 1)) * lda;
    }
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) {
        const int r = col0 + st_r + l * ST_ROWS;
        live_b[l] = r < N;
        pb[l] = B + int64_t(min(r, N - 1)) * ldb;
    }
    uint4 ra[LOADS_A], rb[LOADS_B];
    int cnt_a[LOADS_A], cnt_b[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) cnt_a[l] = 0;
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) cnt_b[l] = 0;
    auto fetch = [&](int kt) {
        const int quad = kt * kMfmaKQ + st_q;
        if (kt < n_full_ktiles) {
#pragma unroll
            for (int l = 0; l < LOADS_A; ++l) ra[l] = load_quad_unchecked<VEC>(pa[l], quad);
#pragma unroll
            for (int l = 0; l < LOADS_B; ++l) rb[l] = load_quad_unchecked<VEC>(pb[l], quad);
        } else {
#pragma unroll
            for (int l = 0; l < LOADS_A; ++l)
                ra[l] = load_quad<VEC>(A, lda, M, kw, tmask, row0 + st_r + l * ST_ROWS, quad);
#pragma unroll
            for (int l = 0; l < LOADS_B; ++l)
                rb[l] = load_quad<VEC>(B, ldb, N, kw, tmask, col0 + st_r + l * ST_ROWS, quad);
        }
    };
    // Writes the fetched quads to LDS and adds their set bits to this thread's row popcounts.
    auto stage = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            const uint4 v = zero_unless(live_a[l], ra[l]);
            cnt_a[l] += popc4(v);
            lds_a[buf][st_q * PLANE_A + st_r + l * ST_ROWS] = v;
        }
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            const uint4 v = zero_unless(live_b[l], rb[l]);
            cnt_b[l] += popc4(v);
            lds_b[buf][st_q * PLANE_B + st_r + l * ST_ROWS] = v;
        }
    };

    v16f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (n_ktiles > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();

    constexpr int kScaleOne = 0x7f7f7f7f;      // E8M0 exponent 127 = scale 1.0 in every byte
    auto word_of = [](const uint4& q, int s) { return s == 0 ? q.x : s == 1 ? q.y : s == 2 ? q.z : q.w; };

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_ktiles) fetch(kt + 1);

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
                for (int i = 0; i < WM; ++i) fa[i] = widen_fp4_a(word_of(aw[i], s));
#pragma unroll
                for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(word_of(bw[j], s));
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                            fa[i], fb[j], acc[i][j], 4 /* A: fp4 */, 4 /* B: fp4 */, 0, kScaleOne, 0, kScaleOne);
            }
        }

        if (kt + 1 < n_ktiles) stage(buf ^ 1);
        __syncthreads();
    }

    // Row popcounts: the kMfmaKQ threads that staged the quads of one row are neighbouring lanes.
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) {
        int c = cnt_a[l];
        c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);       // lane ^ 1
        c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);       // lane ^ 2
        if (st_q == 0) pop_a[st_r + l * ST_ROWS] = 2 * c;
    }
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) {
        int c = cnt_b[l];
        c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);
        c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);
        if (st_q == 0) pop_b[st_r + l * ST_ROWS] = 2 * c;
    }
    __syncthreads();

    // Accumulator register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its 32x32 block.
    // pop_a / pop_b hold twice the popcounts from here on.
    if (!FUSED) {
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int nl = wn * 32 * WN + j * 32 + fr;
            const int n = col0 + nl;
            const int base_n = K - pop_b[nl];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int ml = wm * 32 * WM + i * 32 + 8 * vq + 4 * fh;
                    const int4 pa2 = *reinterpret_cast<const int4*>(&pop_a[ml]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int m = row0 + ml + e;
                        const int pa = e == 0 ? pa2.x : e == 1 ? pa2.y : e == 2 ? pa2.z : pa2.w;
                        const int dot = base_n - pa + 4 * int(acc[i][j][4 * vq + e]);
                        if (m < M && n < N) C[int64_t(m) * ldc + n] = dot;
                    }
                }
        }
    } else {
        // bit(m, n) = (dot >= thr[n]) XOR flip[n] with dot = K - 2pa - 2pb + 4S, i.e.
        // S >= ceil((thr - K + 2pb + 2pa) / 4) = (thr - K + 2pb + 3 + 2pa) >> 2.
        // A ballot over one accumulator register gives, in its low half, the 32-column word of
        // the row held by lanes 0-31 and, in its high half, that of the row 4 below.  The words
        // of one 32-row block are gathered with v_writelane so that lane r (block j = 0) and
        // lane 32 + r (block j = 1) end up holding row r's two words: one store per block row.
        static_assert(WN == 2, "the fused epilogue pairs the two column blocks with the two lane halves");
        int u3[WN];
        uint64_t flip_mask[WN], live_mask[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int nl = wn * 32 * WN + j * 32 + fr;
            const int n = col0 + nl;
            const bool live = n < N;
            const int thr = live ? bn.thr[n] : 0;
            const bool flip = live && ((bn.flip_bits[n >> 5] >> (n & 31)) & 1u) != 0u;
            u3[j] = thr - K + pop_b[nl] + 3;
            flip_mask[j] = __ballot(flip);
            live_mask[j] = __ballot(live);
        }
        const int64_t nw = (int64_t(N) + 31) >> 5;
        const int64_t w = ((int64_t(col0) + wn * 32 * WN) >> 5) + fh;       // word column of this lane
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            int words = 0;
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const int ml = wm * 32 * WM + i * 32 + 8 * vq + 4 * fh;
                const int4 pa2 = *reinterpret_cast<const int4*>(&pop_a[ml]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int pa = e == 0 ? pa2.x : e == 1 ? pa2.y : e == 2 ? pa2.z : pa2.w;
#pragma unroll
                    for (int j = 0; j < WN; ++j) {
                        const bool p = int(acc[i][j][4 * vq + e]) >= ((u3[j] + pa) >> 2);
                        const uint64_t mask = (__ballot(p) ^ flip_mask[j]) & live_mask[j];
                        words = bnn_llvm_writelane(int(uint32_t(mask)), 32 * j + 8 * vq + e, words);
                        words = bnn_llvm_writelane(int(uint32_t(mask >> 32)), 32 * j + 8 * vq + 4 + e, words);
                    }
                }
            }
            const int m = row0 + wm * 32 * WM + i * 32 + fr;
            if (m < M && w < nw) bn.out[int64_t(m) * bn.ld_out + w] = uint32_t(words);
        }
    }
}

template <bool FUSED>
static int launch_mfma(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc,
                       int64_t M, int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    constexpr int WM = 4, WN = 2;
    const int64_t tiles_m = ceil_div(M, 64 * WM), tiles_n = ceil_div(N, 64 * WN);
    if (tiles_m * tiles_n > kMaxDim) return BNN_ERR_UNSUPPORTED;
    const bool vec = aligned_to(A, 16) && aligned_to(B, 16) && lda % 4 == 0 && ldb % 4 == 0;
    const dim3 grid{unsigned(tiles_m * tiles_n)};
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (vec)
        hipLaunchKernelGGL((xnor_gemm_mfma_kernel<WM, WN, true, FUSED>), grid, dim3(256), 0, s, A, lda, B, ldb, C,
                           ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn);
    else
        hipLaunchKernelGGL((xnor_gemm_mfma_kernel<WM, WN, false, FUSED>), grid, dim3(256), 0, s, A, lda, B, ldb,
                           C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn);
    return check_launch();
}

// Entry points used by the dispatcher in xnor_gemm.hip.  The caller has validated the arguments.
bool mfma_path_supports(int64_t K) { return K <= kMfmaMaxK; }

int launch_xnor_gemm_mfma(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                          int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    return launch_mfma<false>(A, lda, B, ldb, C, ldc, M, N, K, BnSignArgs{}, stream);
}

int launch_xnor_gemm_mfma_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    return launch_mfma<true>(A, lda, B, ldb, nullptr, 0, M, N, K, bn, stream);
}

}  // namespace bnn
