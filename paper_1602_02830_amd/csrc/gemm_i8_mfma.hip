// bnn_gemm_i8_mfma: the same +-1 product as the XNOR-popcount kernel, run on
// the dense matrix engine instead (the role the vendor GEMM plays in Sec. 4 /
// Fig. 3 of the paper): +-1 stored as int8, v_mfma_i32_32x32x32_i8, int32
// accumulation.
//
//   C[m][n] = sum_k A[m][k] * B[n][k]          (both operands K-contiguous)
//
// Workgroup = 256 threads = 4 wavefronts in a 2 x 2 arrangement; each
// wavefront owns a (32*WM) x (32*WN) block of the tile as WM x WN MFMA
// accumulators.  Operand tiles of KT = 64 bytes per row are staged
// global -> registers -> LDS (double buffered) and read back as 128-bit LDS
// loads: lane l of a fragment takes row (l % 32), bytes [16*(l/32), +16) of the
// 32-deep K step.  A and B fragments use the same lane -> k assignment, so the
// sum over k is complete whatever order the hardware consumes them in.
// LDS holds one plane of 16-byte slots per 16-byte chunk of the K-tile (slot r =
// that chunk of tile row r), so a fragment read is 32 consecutive slots; two pad
// slots per plane keep the four chunks a row's staging threads write in
// different banks.
//
// bnn_unpack_i8 expands packed bits to this operand format.
#include "bnn_internal.h"

namespace bnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kI8KT = 64;                 // bytes of K per staged tile
constexpr int kI8Chunks = kI8KT / 16;     // 16-byte chunks per tile row

// 16 bytes of row `row` starting at byte k0 of the matrix row; zero outside
// the matrix and for k >= K.
__device__ inline v4i load_chunk_i8(const int8_t* __restrict__ P, int64_t ld, int rows, int K, int row,
                                    int k0) {
    v4i v = {0, 0, 0, 0};
    if (row < rows && k0 < K) {
        v = *reinterpret_cast<const v4i*>(P + int64_t(row) * ld + k0);
        const int valid = K - k0;          // bytes of this chunk that exist
        if (valid < 16) {
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                const int vb = valid - 4 * d;          // valid bytes in dword d
                const uint32_t m = vb >= 4 ? 0xFFFFFFFFu : (vb <= 0 ? 0u : ((1u << (8 * vb)) - 1u));
                v[d] = int(uint32_t(v[d]) & m);
            }
        }
    }
    return v;
}

template <int WM, int WN>
__global__ __launch_bounds__(256) void gemm_i8_mfma_kernel(
    const int8_t* __restrict__ A, int64_t lda, const int8_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n) {
    constexpr int BM = 64 * WM, BN = 64 * WN;
    constexpr int LOADS_A = BM * kI8Chunks / 256, LOADS_B = BN * kI8Chunks / 256;
    constexpr int PLANE_A = BM + 2, PLANE_B = BN + 2;      // slots per chunk plane
    __shared__ v4i lds_a[2][kI8Chunks * PLANE_A];
    __shared__ v4i lds_b[2][kI8Chunks * PLANE_B];

    // Consecutive workgroups go to different dies; give each die a contiguous
    // range of tiles so its L2 keeps a few operand panels.
    int bid = blockIdx.x;
    {
        const int total = tiles_m * tiles_n, per = total / 8;
        if (bid < per * 8) bid = (bid % 8) * per + bid / 8;
    }
    const int tile_m = bid / tiles_n, tile_n = bid - tile_m * tiles_n;
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;       // wavefront position inside the tile
    const int fr = lane & 31, fk = lane >> 5;      // fragment row / K half owned by this lane

    const int st_c = tid % kI8Chunks, st_r = tid / kI8Chunks;
    constexpr int ST_ROWS = 256 / kI8Chunks;
    v4i ra[LOADS_A], rb[LOADS_B];
    auto fetch = [&](int kt) {
        const int k0 = kt * kI8KT + st_c * 16;
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l)
            ra[l] = load_chunk_i8(A, lda, M, K, row0 + st_r + l * ST_ROWS, k0);
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l)
            rb[l] = load_chunk_i8(B, ldb, N, K, col0 + st_r + l * ST_ROWS, k0);
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) lds_a[buf][st_c * PLANE_A + st_r + l * ST_ROWS] = ra[l];
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) lds_b[buf][st_c * PLANE_B + st_r + l * ST_ROWS] = rb[l];
    };

    v16i acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int n_ktiles = (K + kI8KT - 1) / kI8KT;
    if (n_ktiles > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_ktiles) fetch(kt + 1);
#pragma unroll
        for (int ks = 0; ks < kI8KT / 32; ++ks) {
            v4i a[WM], b[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i)
                a[i] = lds_a[buf][(ks * 2 + fk) * PLANE_A + wm * 32 * WM + i * 32 + fr];
#pragma unroll
            for (int j = 0; j < WN; ++j)
                b[j] = lds_b[buf][(ks * 2 + fk) * PLANE_B + wn * 32 * WN + j * 32 + fr];
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < n_ktiles) stage(buf ^ 1);
        __syncthreads();
    }

    // Accumulator register v of lane l is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its 32x32 block.
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int n = col0 + wn * 32 * WN + j * 32 + fr;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = row0 + wm * 32 * WM + i * 32 + 8 * (v / 4) + 4 * fk + (v % 4);
                if (m < M && n < N) store_result(&C[int64_t(m) * ldc + n], acc[i][j][v]);
            }
        }
}

__global__ __launch_bounds__(256) void unpack_i8_kernel(const uint32_t* __restrict__ in, int64_t ld_in,
                                                        int64_t rows, int64_t K, int8_t* __restrict__ out,
                                                        int64_t ld_out, int64_t quads_per_row,
                                                        int64_t n_quads) {
    // One thread per 4 output bytes (ld_out % 4 == 0 on this path).
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < n_quads;
         u += int64_t(gridDim.x) * blockDim.x) {
        const int64_t r = u / quads_per_row;
        const int64_t k0 = (u - r * quads_per_row) * 4;
        uint32_t packed = 0u;
        if (k0 < K) {
            const uint32_t nib = (in[r * ld_in + (k0 >> 5)] >> (k0 & 31)) & 0xFu;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                uint32_t byte = ((nib >> e) & 1u) ? 0x01u : 0xFFu;
                if (k0 + e >= K) byte = 0u;
                packed |= byte << (8 * e);
            }
        }
        *reinterpret_cast<uint32_t*>(out + r * ld_out + k0) = packed;
    }
}

}  // namespace bnn

extern "C" int bnn_gemm_i8_mfma(const int8_t* A, int64_t lda, const int8_t* B, int64_t ldb, int32_t* C,
                                int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    using namespace bnn;
    if (M < 0 || N < 0 || K < 0 || M > kMaxDim || N > kMaxDim || K > kMaxK) return BNN_ERR_INVALID_ARG;
    if (lda < K || ldb < K || ldc < N) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!C || (K > 0 && (!A || !B))) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(C, 4)) return BNN_ERR_ALIGNMENT;
    if (K > 0 && (!aligned_to(A, 16) || !aligned_to(B, 16) || lda % 16 != 0 || ldb % 16 != 0))
        return BNN_ERR_ALIGNMENT;
    constexpr int WM = 4, WN = 2;
    const int64_t tiles_m = ceil_div(M, 64 * WM), tiles_n = ceil_div(N, 64 * WN);
    if (tiles_m * tiles_n > kMaxDim) return BNN_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((gemm_i8_mfma_kernel<WM, WN>), dim3(unsigned(tiles_m * tiles_n)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), A, lda, B, ldb, C, ldc, int(M), int(N), int(K),
                       int(tiles_m), int(tiles_n));
    return check_launch();
}

extern "C" int bnn_unpack_i8(const uint32_t* in, int64_t ld_in, int64_t rows, int64_t K, int8_t* out,
                             int64_t ld_out, void* stream) {
    using namespace bnn;
    if (rows < 0 || K < 0 || rows > kMaxDim || K > kMaxK) return BNN_ERR_INVALID_ARG;
    if (ld_in < ceil_div(K, 32) || ld_out < K) return BNN_ERR_INVALID_ARG;
    if (rows == 0 || ld_out == 0) return BNN_OK;
    if (!in || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(in, 4)) return BNN_ERR_ALIGNMENT;
    if (!aligned_to(out, 4) || ld_out % 4 != 0) return BNN_ERR_ALIGNMENT;
    const int64_t quads_per_row = ld_out / 4;
    const int64_t n_quads = rows * quads_per_row;
    int64_t blocks = ceil_div(n_quads, 256);
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(unpack_i8_kernel, dim3(unsigned(blocks)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), in, ld_in, rows, K, out, ld_out, quads_per_row,
                       n_quads);
    return check_launch();
}
