// bnn_xnor_gemm: the XNOR-popcount matrix product of Sec. 4, Eq. (5), i.e. the
// XnorDotProduct of Alg. 4 over whole matrices.
//
//   C[m][n] = K - 2 * sum_w popcount(A[m][w] ^ B[n][w])
//
// which equals 2*popcount(xnor)-K over the K valid bits once the pad bits of
// both operands are masked (done when a tile is staged, never in the inner loop).
//
// The inner step is two full-rate vector-ALU instructions per 32 connections
// and output: v_xor_b32 and v_bcnt_u32_b32 (whose third operand is the running
// accumulator).  The kernels below differ only in how operands reach registers:
//
//   tiled   - BMxBN output tile per 256-thread workgroup, TMxTN accumulators per
//             thread, operand tiles staged global -> registers -> LDS (double
//             buffered, one barrier per K-tile), read back as 128-bit LDS loads.
//   ksplit  - skinny outputs (few columns or few rows): 8 lanes share one row of
//             the long operand and split K; their partial sums are combined
//             with DPP permutes.
//   naive   - one thread per output, for tiny problems and as a cross-check.
#include "bnn_internal.h"
#include "gemm_staging.h"

namespace bnn {

// ----------------------------------------------------------------------------
// naive: one thread per output element
// ----------------------------------------------------------------------------
__global__ __launch_bounds__(256) void xnor_gemm_naive_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K) {
    const int64_t idx = int64_t(blockIdx.x) * blockDim.x + threadIdx.x;
    if (idx >= int64_t(M) * N) return;
    const int m = int(idx / N);
    const int n = int(idx - int64_t(m) * N);
    const int kw = (K + 31) >> 5;
    const uint32_t* a = A + m * lda;
    const uint32_t* b = B + n * ldb;
    uint32_t acc = 0;
    for (int w = 0; w + 1 < kw; ++w) acc += __popc(a[w] ^ b[w]);
    if (kw > 0) acc += __popc((a[kw - 1] ^ b[kw - 1]) & tail_mask(K));
    C[m * ldc + n] = K - 2 * int(acc);
}

// ----------------------------------------------------------------------------
// tiled: LDS-staged, register-blocked
// ----------------------------------------------------------------------------
// Workgroup = 256 threads = 16 (tx) x 16 (ty).  Thread (ty,tx) owns rows
// ty + 16*i (i < TM) and columns tx + 16*j (j < TN) of the BM x BN tile, with
// BM = 16*TM, BN = 16*TN.  A wavefront is 4 consecutive ty x all 16 tx, so an
// LDS read of an A row is a 16-lane broadcast and the 16 B rows read by one
// instruction are 16 consecutive 16-byte slots: both conflict-free.
//
// LDS holds, per operand and buffer, KQ planes of (rows + 2) 16-byte slots;
// plane q, slot r = words [4q, 4q+4) of tile row r.  The 2-slot pad staggers
// the planes so that the staging stores of 8 consecutive lanes (2 rows x 4
// planes) fall in distinct bank groups.
template <int TM, int TN, int KT>
struct TileCfg {
    static constexpr int BM = 16 * TM;
    static constexpr int BN = 16 * TN;
    static constexpr int KQ = KT / 4;                  // 128-bit quads per K-tile
    static constexpr int PLANE_A = BM + 2;             // slots per plane
    static constexpr int PLANE_B = BN + 2;
    static constexpr int SLOTS_A = KQ * PLANE_A;
    static constexpr int SLOTS_B = KQ * PLANE_B;
    static constexpr int LOADS_A = BM * KQ / 256;      // 16-byte loads per thread per K-tile
    static constexpr int LOADS_B = BN * KQ / 256;
    static_assert(BM * KQ % 256 == 0 && BN * KQ % 256 == 0, "tile must divide among 256 threads");
};

// Three workgroups per compute unit (3 wavefronts per SIMD) keep the vector ALU fed while
// other wavefronts wait on LDS; the bound caps the kernel at 168 VGPRs.
template <int TM, int TN, int KT, bool VEC, bool FUSED>
__global__ __launch_bounds__(256, 3) void xnor_gemm_tiled_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn) {
    using Cfg = TileCfg<TM, TN, KT>;
    __shared__ uint4 lds_a[2][Cfg::SLOTS_A];
    __shared__ uint4 lds_b[2][Cfg::SLOTS_B];

    int tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int row0 = tile_m * Cfg::BM;
    const int col0 = tile_n * Cfg::BN;

    const int tid = threadIdx.x;
    const int tx = tid & 15;
    const int ty = tid >> 4;
    const int kw = (K + 31) >> 5;
    const uint32_t tmask = tail_mask(K);
    const int n_ktiles = (kw + KT - 1) / KT;

    // Staging assignment: load l of this thread covers tile row (tid / KQ) + l * (256 / KQ), plane tid % KQ.
    const int st_q = tid % Cfg::KQ;
    const int st_r = tid / Cfg::KQ;
    constexpr int ST_ROWS = 256 / Cfg::KQ;

    // K-tiles whose every word is complete and unmasked take branch-free loads (row index
    // clamped into the matrix, result zeroed at staging if the row does not exist); only the
    // last, partial K-tile goes through the checked, masking loader.
    const int n_full_ktiles = (K >> 5) / KT;
    const uint32_t* pa[Cfg::LOADS_A];
    const uint32_t* pb[Cfg::LOADS_B];
    bool live_a[Cfg::LOADS_A], live_b[Cfg::LOADS_B];
#pragma unroll
    for (int l = 0; l < Cfg::LOADS_A; ++l) {
        const int r = row0 + st_r + l * ST_ROWS;
        live_a[l] = r < M;
        pa[l] = A + int64_t(min(r, M - 1)) * lda;
    }
#pragma unroll
    for (int l = 0; l < Cfg::LOADS_B; ++l) {
        const int r = col0 + st_r + l * ST_ROWS;
        live_b[l] = r < N;
        pb[l] = B + int64_t(min(r, N - 1)) * ldb;
    }
    uint4 ra[Cfg::LOADS_A], rb[Cfg::LOADS_B];
    auto fetch = [&](int kt) {
        const int quad = kt * Cfg::KQ + st_q;
        if (kt < n_full_ktiles) {
#pragma unroll
            for (int l = 0; l < Cfg::LOADS_A; ++l) ra[l] = load_quad_unchecked<VEC>(pa[l], quad);
#pragma unroll
            for (int l = 0; l < Cfg::LOADS_B; ++l) rb[l] = load_quad_unchecked<VEC>(pb[l], quad);
        } else {
#pragma unroll
            for (int l = 0; l < Cfg::LOADS_A; ++l)
                ra[l] = load_quad<VEC>(A, lda, M, kw, tmask, row0 + st_r + l * ST_ROWS, quad);
#pragma unroll
            for (int l = 0; l < Cfg::LOADS_B; ++l)
                rb[l] = load_quad<VEC>(B, ldb, N, kw, tmask, col0 + st_r + l * ST_ROWS, quad);
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int l = 0; l < Cfg::LOADS_A; ++l)
            lds_a[buf][st_q * Cfg::PLANE_A + st_r + l * ST_ROWS] = zero_unless(live_a[l], ra[l]);
#pragma unroll
        for (int l = 0; l < Cfg::LOADS_B; ++l)
            lds_b[buf][st_q * Cfg::PLANE_B + st_r + l * ST_ROWS] = zero_unless(live_b[l], rb[l]);
    };

    uint32_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = 0u;

    if (n_ktiles > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_ktiles) fetch(kt + 1);   // global loads in flight during the compute below

#pragma unroll 1
        for (int q = 0; q < Cfg::KQ; ++q) {
            uint4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = lds_a[buf][q * Cfg::PLANE_A + ty + 16 * i];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = lds_b[buf][q * Cfg::PLANE_B + tx + 16 * j];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    acc[i][j] += __popc(a[i].x ^ b[j].x);
                    acc[i][j] += __popc(a[i].y ^ b[j].y);
                    acc[i][j] += __popc(a[i].z ^ b[j].z);
                    acc[i][j] += __popc(a[i].w ^ b[j].w);
                }
        }

        if (kt + 1 < n_ktiles) stage(buf ^ 1);
        __syncthreads();
    }

    if (!FUSED) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int m = row0 + ty + 16 * i;
            if (m < M) {
                int32_t* crow = C + int64_t(m) * ldc;
#pragma unroll
                for (int j = 0; j < TN; ++j) {
                    const int n = col0 + tx + 16 * j;
                    if (n < N) store_result(crow + n, K - 2 * int(acc[i][j]));
                }
            }
        }
    } else {
        // bit(m, n) = (K - 2*acc >= thr[n]) XOR flip[n].  Column tx + 16*j of this lane is bit
        // (tx + 16*(j&1)) of word j/2 of the tile row, so a wavefront ballot over column slot j
        // holds, in its 16-bit field q, the half word of tile row 4*wave + q + 16*i.
        static_assert(TN % 2 == 0, "a tile row must be whole 32-bit words");
        int thr[TN];
        bool flip[TN], live[TN];
#pragma unroll
        for (int j = 0; j < TN; ++j) {
            const int n = col0 + tx + 16 * j;
            live[j] = n < N;
            thr[j] = live[j] ? bn.thr[n] : 0;
            flip[j] = live[j] ? ((bn.flip_bits[n >> 5] >> (n & 31)) & 1u) != 0u : false;
        }
        const int q = (tid >> 4) & 3;                  // row group of this lane inside its wavefront
        const int64_t nw = (int64_t(N) + 31) >> 5;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            uint32_t mine = 0u;                        // word kept by the lane with tx == word index
#pragma unroll
            for (int jh = 0; jh < TN / 2; ++jh) {
                const bool p0 = live[2 * jh] && ((K - 2 * int(acc[i][2 * jh]) >= thr[2 * jh]) != flip[2 * jh]);
                const bool p1 = live[2 * jh + 1] &&
                                ((K - 2 * int(acc[i][2 * jh + 1]) >= thr[2 * jh + 1]) != flip[2 * jh + 1]);
                const uint64_t m0 = __ballot(p0), m1 = __ballot(p1);
                const uint32_t word = uint32_t((m0 >> (16 * q)) & 0xFFFFu) | (uint32_t((m1 >> (16 * q)) & 0xFFFFu) << 16);
                if (tx == jh) mine = word;
            }
            const int m = row0 + ty + 16 * i;
            const int64_t w = int64_t(tile_n) * (TN / 2) + tx;
            if (tx < TN / 2 && m < M && w < nw) bn.out[int64_t(m) * bn.ld_out + w] = mine;
        }
    }
}

// ----------------------------------------------------------------------------
// ksplit: skinny outputs.  An aligned group of LPR = 8 or 16 lanes owns one row of the long
// operand X and up to 16 rows of the short operand Y; the lanes split K by 16-byte quads (so a
// group reads 128 or 256 contiguous bytes of its X row per load), each lane keeps 16 partial sums,
// and the group combines them with three or four DPP permutes per sum.  K advances in chunks of
// 256 words: the workgroup stages the chunk of Y in LDS (every group needs all of it) while each
// lane's quads of X are in flight, so one chunk costs a single global-memory round trip.  16 lanes
// per row halve the serial work of a lane and double the workgroups (10000 x 10, K = 4096:
// 7.0 -> 5.5 us); the launcher uses them while the grid stays small.  out(x, y) is
// stored at C[x * sx + y * sy], which lets the same kernel serve few columns (X = A) and few
// rows (X = B).
// ----------------------------------------------------------------------------
constexpr int kSkinnyCols = 16;
constexpr int kSkinnyChunkQuads = 64;     // 256 words of K per chunk
constexpr int64_t kKsplitWideMaxGroups = 1024;   // row groups of 16 up to which a row gets 16 lanes

template <bool VEC, int LPR>
__global__ __launch_bounds__(256) void xnor_gemm_ksplit_kernel(
    const uint32_t* __restrict__ X, int64_t ldx, int nx, const uint32_t* __restrict__ Y, int64_t ldy, int ny,
    int32_t* __restrict__ C, int64_t sx, int64_t sy, int K) {
    __shared__ uint4 lds_y[kSkinnyCols * kSkinnyChunkQuads];          // [row][quad]
    const int tid = threadIdx.x;
    static_assert(LPR == 8 || LPR == 16, "aligned groups of 8 or 16 lanes per row");
    constexpr int ROWS = 256 / LPR;                                   // rows (lane groups) per workgroup
    constexpr int STEPS = kSkinnyChunkQuads / LPR;                    // quads per lane and chunk
    const int q = tid & (LPR - 1);
    const int row = blockIdx.x * ROWS + tid / LPR;
    const int y0 = blockIdx.y * kSkinnyCols;
    const int kw = (K + 31) >> 5;
    const uint32_t tmask = tail_mask(K);
    const int n_quads = (kw + 3) >> 2;
    const bool live = row < nx;
    const int xr = min(row, nx - 1);

    int acc[kSkinnyCols];
#pragma unroll
    for (int j = 0; j < kSkinnyCols; ++j) acc[j] = 0;

    // Quads made of complete, unmasked words are loaded without any check (index clamped into that
    // range, result zeroed afterwards if the quad does not exist): the loads of a chunk then carry no
    // control flow and are all in flight together.  The one quad that may be partial or hold pad
    // bits (index n_full) goes through the checked, masking loader, once per chunk that contains it.
    const int n_full = (K >> 5) >> 2;
    const uint32_t* xrow = X + int64_t(xr) * ldx;

    for (int q0 = 0; q0 < n_quads; q0 += kSkinnyChunkQuads) {
        // This lane's quads of the chunk: q, q + LPR, q + 2*LPR, ... (zero beyond the row's end).
        uint4 a[STEPS] = {};
        if (n_full > 0) {
#pragma unroll
            for (int t = 0; t < STEPS; ++t)
                a[t] = load_quad_unchecked<VEC>(xrow, min(q0 + q + LPR * t, n_full - 1));
        }
        const bool tail_here = n_full < n_quads && n_full >= q0 && n_full < q0 + kSkinnyChunkQuads;
        uint4 a_tail = make_uint4(0u, 0u, 0u, 0u);
        if (tail_here) a_tail = load_quad<VEC>(X, ldx, nx, kw, tmask, xr, n_full);
        // Stage Y: 16 rows x 64 quads, 4 quads per thread; rows beyond ny repeat the last row.
        uint4 yv[kSkinnyCols * kSkinnyChunkQuads / 256] = {};
        if (n_full > 0) {
#pragma unroll
            for (int t = 0; t < kSkinnyCols * kSkinnyChunkQuads / 256; ++t) {
                const int idx = tid + 256 * t;
                const int yr = idx / kSkinnyChunkQuads, yq = idx % kSkinnyChunkQuads;
                yv[t] = load_quad_unchecked<VEC>(Y + int64_t(min(y0 + yr, ny - 1)) * ldy, min(q0 + yq, n_full - 1));
            }
        }
        __syncthreads();                                              // previous chunk fully consumed
#pragma unroll
        for (int t = 0; t < kSkinnyCols * kSkinnyChunkQuads / 256; ++t) {
            const int idx = tid + 256 * t;
            const int yr = idx / kSkinnyChunkQuads, yq = idx % kSkinnyChunkQuads;
            uint4 v = zero_unless(n_full > 0 && q0 + yq < n_full, yv[t]);
            if (tail_here && q0 + yq == n_full) v = load_quad<VEC>(Y, ldy, ny, kw, tmask, min(y0 + yr, ny - 1), n_full);
            lds_y[idx] = v;
        }
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            const int qi = q0 + q + LPR * t;
            a[t] = zero_unless(n_full > 0 && qi < n_full, a[t]);
            if (qi == n_full) a[t] = a_tail;
        }
        __syncthreads();
        // Steps and columns that do not exist are skipped (both bounds are wavefront-uniform).
        const int steps = (min(kSkinnyChunkQuads, n_quads - q0) + LPR - 1) / LPR;
        const int cols = min(kSkinnyCols, ny - y0);
#pragma unroll
        for (int t = 0; t < STEPS; ++t) {
            if (t < steps) {
#pragma unroll
                for (int j = 0; j < kSkinnyCols; ++j) {
                    if (j < cols) {
                        const uint4 b = lds_y[j * kSkinnyChunkQuads + q + LPR * t];
                        acc[j] += __popc(a[t].x ^ b.x) + __popc(a[t].y ^ b.y) + __popc(a[t].z ^ b.z) +
                                  __popc(a[t].w ^ b.w);
                    }
                }
            }
        }
    }
#pragma unroll
    for (int j = 0; j < kSkinnyCols; ++j) {
        int v = acc[j];
        v += __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true);    // lane ^ 1
        v += __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true);    // lane ^ 2
        v += __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true);   // other quad of the 8 lanes
        if (LPR == 16) v += __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true);   // other 8 lanes of the 16
        acc[j] = v;
    }
    // Lane q of the group stores columns q, q + LPR, ... below 16.
#pragma unroll
    for (int h = 0; h < kSkinnyCols / LPR; ++h) {
        const int j = q + LPR * h;
        int v = 0;
#pragma unroll
        for (int jj = 0; jj < kSkinnyCols; ++jj) v = (jj == j) ? acc[jj] : v;
        if (live && y0 + j < ny) C[int64_t(row) * sx + int64_t(y0 + j) * sy] = K - 2 * v;
    }
}

// ----------------------------------------------------------------------------
// host side
// ----------------------------------------------------------------------------
enum { KERNEL_AUTO = 0, KERNEL_NAIVE = 1, KERNEL_TILED128 = 2, KERNEL_KSPLIT = 3, KERNEL_TILED64 = 4,
       KERNEL_MFMA = 5, KERNEL_MFMA128 = 6, KERNEL_MFMA_SHORTK = 7, KERNEL_MFMA_PERSIST = 8,
       KERNEL_MFMA_BIG = 9, KERNEL_MFMA_SPLITK = 10, KERNEL_LAST = KERNEL_MFMA_SPLITK };

// Matrix-engine variant, defined in xnor_gemm_mfma.hip.
bool mfma_path_supports(int64_t K);
int launch_xnor_gemm_mfma(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                          int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream);
int launch_xnor_gemm_mfma_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                int64_t N, int64_t K, BnSignArgs bn, void* stream);
int launch_xnor_gemm_mfma128(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                             int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream);
int launch_xnor_gemm_mfma128_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                   int64_t N, int64_t K, BnSignArgs bn, void* stream);
// Whole-tile form of the 256 x 128 matrix-engine kernel (xnor_gemm_mfma_persist.hip), launched as a tile walk
// (walk: one workgroup per resident slot) or with one workgroup per tile: BNN_ERR_UNSUPPORTED, with nothing
// launched, for the products it does not take.
int launch_xnor_gemm_mfma_persist(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                  int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, bool walk, BnSignArgs bn,
                                  void* stream);
int64_t mfma_persist_slots();
bool mfma_persist_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t ldc, int64_t M,
                           int64_t N, int64_t K, bool fused, bool walk);
// 256 x 256-tile form of the fused product for one wavefront per SIMD (xnor_gemm_mfma_big.hip), one workgroup
// per compute unit: BNN_ERR_UNSUPPORTED, with nothing launched, for the products it does not take.
int launch_xnor_gemm_mfma_big(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                              int64_t K, BnSignArgs bn, void* stream);
bool mfma_big_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                       int64_t K, const BnSignArgs& bn);
bool mfma_big_prefers(int64_t M, int64_t N);
// 32 x 32 output tiles with K split over the wavefronts of a workgroup (xnor_gemm_mfma_splitk.hip), for small
// outputs with a long K: BNN_ERR_UNSUPPORTED, with nothing launched, for the products it does not take.
bool mfma_splitk_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                          int64_t K);
int launch_xnor_gemm_mfma_splitk(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                 int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, const BnSignArgs& bn,
                                 void* stream);
// Short-K organisation of the matrix-engine kernel, defined in xnor_gemm_mfma_shortk.hip.
bool mfma_shortk_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t K);
int launch_xnor_gemm_mfma_shortk(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                 int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream);
int launch_xnor_gemm_mfma_shortk_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                       int64_t N, int64_t K, BnSignArgs bn, void* stream);
bool mfma_planes_path_supports(int64_t K);
int launch_bitplane_gemm_mfma(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int32_t* C,
                              int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream);
int launch_bitplane_gemm_mfma_fused(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int64_t M,
                                    int64_t N, int64_t K, BnSignArgs bn, void* stream);
// Vector-ALU form for 255 * K beyond the matrix engine's exact range, defined in valu_fallbacks.hip.
int launch_bitplane_gemm_valu(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int32_t* C,
                              int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, BnSignArgs bn, void* stream);

template <int TM, int TN, int KT, bool FUSED>
static void launch_tiled(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                         int64_t ldc, int M, int N, int K, BnSignArgs bn, hipStream_t s) {
    using Cfg = TileCfg<TM, TN, KT>;
    const int tiles_m = int(ceil_div(M, Cfg::BM));
    const int tiles_n = int(ceil_div(N, Cfg::BN));
    const bool vec = aligned_to(A, 16) && aligned_to(B, 16) && lda % 4 == 0 && ldb % 4 == 0;
    const dim3 grid(unsigned(int64_t(tiles_m) * tiles_n));
    if (vec)
        hipLaunchKernelGGL((xnor_gemm_tiled_kernel<TM, TN, KT, true, FUSED>), grid, dim3(256), 0, s, A, lda,
                           B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, bn);
    else
        hipLaunchKernelGGL((xnor_gemm_tiled_kernel<TM, TN, KT, false, FUSED>), grid, dim3(256), 0, s, A, lda,
                           B, ldb, C, ldc, M, N, K, tiles_m, tiles_n, bn);
}

// Kernel choice, from measurements on MI355X: the matrix-engine kernels are 2-4x faster than the
// vector-ALU XNOR-popcount kernels down to a few dozen tiles.  Their 256 x 128 tile (two workgroups
// per compute unit) wins for long K on a grid of a thousand tiles or more; otherwise the
// 128 x 128 tile (three workgroups per compute unit) hides short K loops better.  For K up to 1152
// on a grid that fills the chip, the short-K organisation (B tile resident, several A tiles per
// workgroup, only the K words that exist) is 5-25 % faster still; it needs operands that allow
// 16-byte loads (short_ok).  Tiny grids go to the
// 64 x 64 XNOR tiles, which spread over more compute units; skinny outputs go to the K-split kernel;
// K beyond the exact-fp32 range stays on the vector ALU.
//
// The 256 x 128 kernel as a tile walk (kernel 8; walk_ok: the product is one it takes, which includes
// more tiles than the chip's resident slots) against one workgroup per tile, kernel time in us, N = 4096:
// the walk wins where the last round of tiles is partial (every compute unit gets the same share of it:
// fused M = 10000, K = 4096 57.5 -> 55.5, M = 6144 36.6 -> 35.6; int32 M = 9216, K = 2048 41.3 -> 39.1) and
// loses where the tiles fill whole rounds or run for many rounds (the hardware hands a tile to whichever
// slot frees up first: fused 8192^3 167 vs 173, int32 M = 32768, K = 4096 209 vs 214); at 1.25 rounds with
// the fused epilogue the 128 x 128 tiles win (M = 5120, K = 4096: 32.2 vs 35.1).
// With int32 output the 256 x 128 kernel (in its whole-tile form where the product allows it) also takes
// shorter K and smaller grids than with the fused epilogue, its 128 KB of stores per tile being the larger
// part of a tile's life: K = 2048, M = 12288 55.0 vs 59.8 (128 x 128 tiles), but M = 8192 42.5 vs 40.0.
// (whole_ok: the product is one the whole-tile form takes.)
//
// The 256 x 256-tile kernel for one wavefront per SIMD (kernel 9, fused products only; big_ok: the product is
// one it takes) against the choices above, 121 shapes with N = 1024 .. 8192, K = 2048 .. 8192, M = 4096 .. 65536:
// 10 - 20 % faster wherever a compute unit's row strip has 512 rows or more, or exactly 256
// (10000 x 4096 x 4096 55.7 -> 51.5 us, 8192^3 167 -> 151, 16384 x 4096 x 4096 88.6 -> 77, 65536 x 1024 x 8192
// 169 -> 147); with 257 .. 511 rows a strip is one tile and a bit, and the second start-up costs what the
// kernel gains (20000 x 1024 x 2048 19.3 vs 21.0, 10000 x 2048 x 4096 32.8 vs 33.1).
static int choose_kernel(int64_t M, int64_t N, int64_t K, bool fused, bool short_ok, bool whole_ok, bool walk_ok,
                         bool big_ok, bool splitk_ok) {
    // Small outputs: 32 x 32 tiles with K split inside the workgroup, while the tiles are few enough for the
    // workgroup dispatch rate.  Launches replayed from a graph, fused, against the choice below:
    // 256 x 1024 (256 tiles) K = 512 3.3 vs 3.6 us, 1024 3.7 vs 4.2, 8192 5.3 vs 12.9, 16384 8.1 vs 23.0;
    // 512 x 1024 (512 tiles) K = 1024 4.7 vs 4.2, 2048 4.7 vs 5.5, 8192 7.1 vs 12.9;
    // 1024 x 1024 (1024 tiles) K = 2048 6.7 vs 5.5, 4096 6.8 vs 8.0, 16384 19.3 vs 23.2.  The int32 form alike,
    // skinny outputs included (against the lane-group kernel below: 10000 x 10, K = 4096, 4.3 vs 5.1 us,
    // 16384 x 16 4.6 vs 6.8, 1 x 4096 3.2 vs 3.6, 4 x 1024, K = 8192, 4.6 vs 4.3).
    if (splitk_ok) {
        const int64_t tiles32 = ceil_div(M, 32) * ceil_div(N, 32);
        if (tiles32 <= 256 || (tiles32 <= 512 && K >= 2048) || (tiles32 <= 1024 && K >= 4096))
            return KERNEL_MFMA_SPLITK;
    }
    if (!fused && (N <= 16 || M <= 4)) return KERNEL_KSPLIT;
    if (fused && big_ok && mfma_big_prefers(M, N)) return KERNEL_MFMA_BIG;
    const int64_t tiles128 = ceil_div(M, 128) * ceil_div(N, 128);
    const int64_t tiles256 = ceil_div(M, 256) * ceil_div(N, 128);
    if (mfma_path_supports(K)) {
        if (walk_ok) {
            const int64_t slots = mfma_persist_slots(), rem = tiles256 % slots;
            const bool partial_round = rem >= slots / 8 && rem <= slots - slots / 8;
            if (!fused && partial_round) return KERNEL_MFMA_PERSIST;
            if (fused && K >= 2048 && partial_round && 2 * tiles256 >= 3 * slots) return KERNEL_MFMA_PERSIST;
        }
        if (!fused && whole_ok && K * tiles256 >= int64_t(4096) * 768) return KERNEL_MFMA;
        if (K >= 4096 && tiles256 >= 1024) return KERNEL_MFMA;
        // fused, K = 2048, N = 4096: M = 8192 27.4 vs 28.0 (128 x 128 tiles), 12288 39.4 vs 40.7, 20000 62.4 vs 65.5
        if (fused && K >= 2048 && tiles256 >= 768) return KERNEL_MFMA;
        if (short_ok && tiles128 >= 768) return KERNEL_MFMA_SHORTK;
        // Small grids, measured against the 64 x 64 vector-ALU tiles (kernel time, fused / int32):
        // 64 x 1024 x 1024 5.4 vs 6.8 / 7.2 vs 5.8 us, 256 x 1024 x 8192 17.2 vs 26.3 / 18.7 vs 24.6 us,
        // 512 x 512 x 2048 7.2 vs 9.6 / 8.7 vs 8.5 us: the fused form always wins on the matrix engine,
        // the int32 form once K is long.
        if (fused || tiles128 >= 32 || K >= 4096) return KERNEL_MFMA128;
    }
    return tiles128 >= 512 ? KERNEL_TILED128 : KERNEL_TILED64;
}

static int xnor_gemm_dispatch(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                              int64_t ldc, int64_t M, int64_t N, int64_t K, int kernel_id,
                              void* stream) {
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return BNN_ERR_INVALID_ARG;
    if (kernel_id < KERNEL_AUTO || kernel_id > KERNEL_LAST) return BNN_ERR_INVALID_ARG;
    if ((kernel_id == KERNEL_MFMA || kernel_id == KERNEL_MFMA128 || kernel_id == KERNEL_MFMA_PERSIST ||
         kernel_id == KERNEL_MFMA_BIG) &&
        !mfma_path_supports(K))
        return BNN_ERR_UNSUPPORTED;
    if (kernel_id == KERNEL_MFMA_SHORTK && !mfma_shortk_supports(A, lda, B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    const int64_t kw = ceil_div(K, 32);
    if (lda < kw || ldb < kw || ldc < N) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!C || (K > 0 && (!A || !B))) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(A, 4) || !aligned_to(B, 4) || !aligned_to(C, 4)) return BNN_ERR_ALIGNMENT;
    // Tile grids and the row / column indices inside a tile (up to one tile past the matrix) are 32-bit.
    if (ceil_div(M, 16) * ceil_div(N, 16) > kMaxDim || M > kMaxDim - 1024 || N > kMaxDim - 1024)
        return BNN_ERR_UNSUPPORTED;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int m = int(M), n = int(N), k = int(K);

    if (kernel_id == KERNEL_AUTO)
        kernel_id = choose_kernel(M, N, K, /*fused=*/false, mfma_shortk_supports(A, lda, B, ldb, K),
                                  mfma_persist_supports(A, lda, B, ldb, ldc, M, N, K, false, false),
                                  mfma_persist_supports(A, lda, B, ldb, ldc, M, N, K, false, true), false,
                                  K >= 512 && mfma_splitk_supports(A, lda, B, ldb, M, N, K));

    switch (kernel_id) {
        case KERNEL_NAIVE: {
            const int64_t total = M * N;
            if (ceil_div(total, 256) > kMaxDim) return BNN_ERR_UNSUPPORTED;
            hipLaunchKernelGGL(xnor_gemm_naive_kernel, dim3(unsigned(ceil_div(total, 256))), dim3(256), 0, s,
                               A, lda, B, ldb, C, ldc, m, n, k);
            break;
        }
        case KERNEL_TILED128:
            launch_tiled<8, 8, 16, false>(A, lda, B, ldb, C, ldc, m, n, k, BnSignArgs{}, s);
            break;
        case KERNEL_TILED64:
            launch_tiled<4, 4, 16, false>(A, lda, B, ldb, C, ldc, m, n, k, BnSignArgs{}, s);
            break;
        case KERNEL_KSPLIT: {
            // The long operand gets one group of 8 lanes per row, the short one 16 rows per pass.
            const bool a_long = M >= N;
            const uint32_t* X = a_long ? A : B;
            const uint32_t* Y = a_long ? B : A;
            const int64_t ldx = a_long ? lda : ldb, ldy = a_long ? ldb : lda;
            const int nx = a_long ? m : n, ny = a_long ? n : m;
            const int64_t sx = a_long ? ldc : 1, sy = a_long ? 1 : ldc;
            const int64_t passes = ceil_div(ny, kSkinnyCols);
            if (passes > 65535) return BNN_ERR_UNSUPPORTED;
            const bool vec = aligned_to(A, 16) && aligned_to(B, 16) && lda % 4 == 0 && ldb % 4 == 0;
            // 16 lanes per row (16 rows per workgroup) while that still gives every compute unit few
            // workgroups: twice the workgroups, half the serial work per lane.
            if (ceil_div(nx, 16) <= kKsplitWideMaxGroups) {
                const dim3 grid(unsigned(ceil_div(nx, 16)), unsigned(passes));
                if (vec)
                    hipLaunchKernelGGL((xnor_gemm_ksplit_kernel<true, 16>), grid, dim3(256), 0, s, X, ldx, nx, Y, ldy,
                                       ny, C, sx, sy, k);
                else
                    hipLaunchKernelGGL((xnor_gemm_ksplit_kernel<false, 16>), grid, dim3(256), 0, s, X, ldx, nx, Y, ldy,
                                       ny, C, sx, sy, k);
            } else {
                const dim3 grid(unsigned(ceil_div(nx, 32)), unsigned(passes));
                if (vec)
                    hipLaunchKernelGGL((xnor_gemm_ksplit_kernel<true, 8>), grid, dim3(256), 0, s, X, ldx, nx, Y, ldy,
                                       ny, C, sx, sy, k);
                else
                    hipLaunchKernelGGL((xnor_gemm_ksplit_kernel<false, 8>), grid, dim3(256), 0, s, X, ldx, nx, Y, ldy,
                                       ny, C, sx, sy, k);
            }
            break;
        }
        case KERNEL_MFMA: {
            // Whole-tile products take the form whose int32 stores go to scalar row bases, one workgroup per tile.
            const int st = launch_xnor_gemm_mfma_persist(A, lda, B, ldb, C, ldc, M, N, K, false, false, BnSignArgs{}, stream);
            if (st != BNN_ERR_UNSUPPORTED) return st;
            return launch_xnor_gemm_mfma(A, lda, B, ldb, C, ldc, M, N, K, stream);
        }
        case KERNEL_MFMA_PERSIST:
            return launch_xnor_gemm_mfma_persist(A, lda, B, ldb, C, ldc, M, N, K, false, true, BnSignArgs{}, stream);
        case KERNEL_MFMA_BIG:
            return BNN_ERR_UNSUPPORTED;          // a kernel of the fused product only
        case KERNEL_MFMA_SPLITK:
            return launch_xnor_gemm_mfma_splitk(A, lda, B, ldb, C, ldc, M, N, K, false, BnSignArgs{}, stream);
        case KERNEL_MFMA128:
            return launch_xnor_gemm_mfma128(A, lda, B, ldb, C, ldc, M, N, K, stream);
        case KERNEL_MFMA_SHORTK:
            return launch_xnor_gemm_mfma_shortk(A, lda, B, ldb, C, ldc, M, N, K, stream);
        default:
            return BNN_ERR_INVALID_ARG;
    }
    return check_launch();
}

static int xnor_gemm_bn_sign_pack_dispatch(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb,
                                           int64_t M, int64_t N, int64_t K, const int32_t* thr,
                                           const uint32_t* flip_bits, uint32_t* out, int64_t ld_out,
                                           int kernel_id, void* stream) {
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return BNN_ERR_INVALID_ARG;
    if (kernel_id != KERNEL_AUTO && kernel_id != KERNEL_TILED128 && kernel_id != KERNEL_TILED64 &&
        kernel_id != KERNEL_MFMA && kernel_id != KERNEL_MFMA128 && kernel_id != KERNEL_MFMA_SHORTK &&
        kernel_id != KERNEL_MFMA_PERSIST && kernel_id != KERNEL_MFMA_BIG && kernel_id != KERNEL_MFMA_SPLITK)
        return BNN_ERR_INVALID_ARG;
    if ((kernel_id == KERNEL_MFMA || kernel_id == KERNEL_MFMA128 || kernel_id == KERNEL_MFMA_PERSIST ||
         kernel_id == KERNEL_MFMA_BIG) &&
        !mfma_path_supports(K))
        return BNN_ERR_UNSUPPORTED;
    if (kernel_id == KERNEL_MFMA_SHORTK && !mfma_shortk_supports(A, lda, B, ldb, K)) return BNN_ERR_UNSUPPORTED;
    const int64_t kw = ceil_div(K, 32);
    if (lda < kw || ldb < kw || ld_out < ceil_div(N, 32)) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!thr || !flip_bits || !out || (K > 0 && (!A || !B))) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(A, 4) || !aligned_to(B, 4) || !aligned_to(thr, 4) || !aligned_to(flip_bits, 4) ||
        !aligned_to(out, 4))
        return BNN_ERR_ALIGNMENT;
    // Tile grids and the row / column indices inside a tile (up to one tile past the matrix) are 32-bit.
    if (ceil_div(M, 16) * ceil_div(N, 16) > kMaxDim || M > kMaxDim - 1024 || N > kMaxDim - 1024)
        return BNN_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const BnSignArgs bn{thr, flip_bits, out, ld_out};
    if (kernel_id == KERNEL_AUTO)
        kernel_id = choose_kernel(M, N, K, /*fused=*/true, mfma_shortk_supports(A, lda, B, ldb, K),
                                  mfma_persist_supports(A, lda, B, ldb, 0, M, N, K, true, false),
                                  mfma_persist_supports(A, lda, B, ldb, 0, M, N, K, true, true),
                                  mfma_big_supports(A, lda, B, ldb, M, N, K, bn),
                                  K >= 512 && mfma_splitk_supports(A, lda, B, ldb, M, N, K));
    if (kernel_id == KERNEL_MFMA_SHORTK) return launch_xnor_gemm_mfma_shortk_fused(A, lda, B, ldb, M, N, K, bn, stream);
    if (kernel_id == KERNEL_MFMA_PERSIST)
        return launch_xnor_gemm_mfma_persist(A, lda, B, ldb, nullptr, 0, M, N, K, true, true, bn, stream);
    if (kernel_id == KERNEL_MFMA_BIG) return launch_xnor_gemm_mfma_big(A, lda, B, ldb, M, N, K, bn, stream);
    if (kernel_id == KERNEL_MFMA_SPLITK)
        return launch_xnor_gemm_mfma_splitk(A, lda, B, ldb, nullptr, 0, M, N, K, true, bn, stream);
    if (kernel_id == KERNEL_MFMA) return launch_xnor_gemm_mfma_fused(A, lda, B, ldb, M, N, K, bn, stream);
    if (kernel_id == KERNEL_MFMA128) return launch_xnor_gemm_mfma128_fused(A, lda, B, ldb, M, N, K, bn, stream);
    if (kernel_id == KERNEL_TILED128)
        launch_tiled<8, 8, 16, true>(A, lda, B, ldb, nullptr, 0, int(M), int(N), int(K), bn, s);
    else
        launch_tiled<4, 4, 16, true>(A, lda, B, ldb, nullptr, 0, int(M), int(N), int(K), bn, s);
    return check_launch();
}

// First layer on 8-bit inputs (Alg. 4 step 1): argument checks shared by the plain and fused calls.
static int bitplane_gemm_check(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int64_t M,
                               int64_t N, int64_t K) {
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return BNN_ERR_INVALID_ARG;
    const int64_t kw = ceil_div(K, 32);
    if (ldx < 8 * kw || ldb < kw) return BNN_ERR_INVALID_ARG;
    if (M > 0 && N > 0 && K > 0 && (!Xp || !B)) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(Xp, 4) || !aligned_to(B, 4)) return BNN_ERR_ALIGNMENT;
    if (255 * K > kMaxK) return BNN_ERR_INVALID_ARG;           // the sums must fit int32
    if (M > kMaxDim - 1024 || N > kMaxDim - 1024) return BNN_ERR_UNSUPPORTED;
    return BNN_OK;
}

}  // namespace bnn

extern "C" int bnn_bitplane_gemm(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int32_t* C,
                                 int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    using namespace bnn;
    const int st = bitplane_gemm_check(Xp, ldx, B, ldb, M, N, K);
    if (st != BNN_OK) return st;
    if (ldc < N) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!C) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(C, 4)) return BNN_ERR_ALIGNMENT;
    if (!mfma_planes_path_supports(K))
        return launch_bitplane_gemm_valu(Xp, ldx, B, ldb, C, ldc, M, N, K, false, BnSignArgs{}, stream);
    return launch_bitplane_gemm_mfma(Xp, ldx, B, ldb, C, ldc, M, N, K, stream);
}

extern "C" int bnn_bitplane_gemm_bn_sign_pack(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb,
                                              int64_t M, int64_t N, int64_t K, const int32_t* thr,
                                              const uint32_t* flip_bits, uint32_t* out, int64_t ld_out,
                                              void* stream) {
    using namespace bnn;
    const int st = bitplane_gemm_check(Xp, ldx, B, ldb, M, N, K);
    if (st != BNN_OK) return st;
    if (ld_out < ceil_div(N, 32)) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!thr || !flip_bits || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(thr, 4) || !aligned_to(flip_bits, 4) || !aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;
    if (!mfma_planes_path_supports(K))
        return launch_bitplane_gemm_valu(Xp, ldx, B, ldb, nullptr, 0, M, N, K, true,
                                         BnSignArgs{thr, flip_bits, out, ld_out}, stream);
    return launch_bitplane_gemm_mfma_fused(Xp, ldx, B, ldb, M, N, K, BnSignArgs{thr, flip_bits, out, ld_out},
                                           stream);
}

extern "C" int bnn_xnor_gemm_bn_sign_pack(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb,
                                          int64_t M, int64_t N, int64_t K, const int32_t* thr,
                                          const uint32_t* flip_bits, uint32_t* out, int64_t ld_out,
                                          void* stream) {
    return bnn::xnor_gemm_bn_sign_pack_dispatch(A, lda, B, ldb, M, N, K, thr, flip_bits, out, ld_out,
                                                bnn::KERNEL_AUTO, stream);
}

extern "C" int bnn_xnor_gemm_bn_sign_pack_kernel(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb,
                                                 int64_t M, int64_t N, int64_t K, const int32_t* thr,
                                                 const uint32_t* flip_bits, uint32_t* out, int64_t ld_out,
                                                 int kernel_id, void* stream) {
    return bnn::xnor_gemm_bn_sign_pack_dispatch(A, lda, B, ldb, M, N, K, thr, flip_bits, out, ld_out, kernel_id,
                                                stream);
}

extern "C" int bnn_xnor_gemm(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                             int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    return bnn::xnor_gemm_dispatch(A, lda, B, ldb, C, ldc, M, N, K, bnn::KERNEL_AUTO, stream);
}

extern "C" int bnn_xnor_gemm_kernel(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb,
                                    int32_t* C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                                    int kernel_id, void* stream) {
    return bnn::xnor_gemm_dispatch(A, lda, B, ldb, C, ldc, M, N, K, kernel_id, stream);
}
