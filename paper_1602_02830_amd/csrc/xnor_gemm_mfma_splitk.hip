// Bits-in, matrix-engine-inside binary product (Sec. 4 Eq. (5), the XnorDotProduct of Alg. 4) for
// small outputs with a long K: the fully connected layers of a network at inference batch sizes
// (in the ConvNet architecture that Sec. 2.2 refers to, at batch 256: 256 x 1024 outputs over
// K = 8192), where 128 x 128 or 256 x 128 output tiles would leave most of the 256 compute units
// without a tile.
//
// A workgroup owns one 32 x 32 output tile, so a 256 x 1024 output is 256 workgroups, and splits K
// over its four wavefronts: of every aligned group of 8 quads (a quad = 4 words = 128 bits of a
// row) wavefront w takes quads 2w and 2w + 1, one per lane half.  Lane (r = lane % 32,
// h = lane / 32) loads its quad of A's row r and of B's row r straight from global memory into
// registers - the operand layout of v_mfma_f32_32x32x64_f8f6f4 is exactly "lane (r, h) holds 32
// consecutive K elements of row r", and the order in which K is summed is free - widens the four
// words to fp4 codes (mfma_fp4.h) and issues four MFMAs.  Nothing is staged in LDS and no barrier
// is met inside the K loop; a lane fetches the next 4 quads of each operand while it multiplies the
// current 4, so the loop exposes one round trip to memory.
//
// The four partial 32 x 32 sums (exact fp32 counts) and the row / column popcounts meet in LDS
// once; wavefront w then finishes accumulator registers 4w .. 4w + 3, i.e. rows 8w + 4h + e of the
// tile: pre-activation K - 2pa - 2pb + 4S, stored as int32, or compared with the folded BatchNorm
// threshold (Alg. 4: Sign(BatchNorm(.)), bn_fold.cpp) and turned into output words by one ballot
// per register (the ballot's two halves are the 32-column words of two rows).
//
// Requirements (checked by the launcher): K a positive multiple of 128 up to 2^24 (exact fp32
// sums), A and B 16-byte aligned, lda and ldb multiples of 4 words.
#include <cstdint>

#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {
namespace splitk {

constexpr int kTile = 32;
constexpr int kWaves = 4;
constexpr int kQuadStride = 2 * kWaves;   // quads between two consecutive quads of one lane
constexpr int kBatch = 4;                 // quads of each operand a lane loads at a time (two such batches in flight)

template <bool FUSED>
__global__ __launch_bounds__(256) void xnor_gemm_mfma_splitk_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn) {
    __shared__ float4 part[kWaves][4][kWave];     // [wavefront][accumulator registers 4g .. 4g+3][lane]
    __shared__ __attribute__((aligned(16))) int pop_part[kWaves][kWave];   // 2*popcount over the wavefront's share of K:
                                                                          // [0, 32) rows of A, [32, 64) rows of B
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int fr = lane & 31, fh = lane >> 5;
    int tm, tn;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tm, tn);
    const int row0 = tm * kTile, col0 = tn * kTile;

    // Rows beyond the matrix repeat its last row; their results are never stored.
    const uint4* a_row = reinterpret_cast<const uint4*>(A + int64_t(min(row0 + fr, M - 1)) * lda);
    const uint4* b_row = reinterpret_cast<const uint4*>(B + int64_t(min(col0 + fr, N - 1)) * ldb);
    const int nq = K >> 7;
    const int first = 2 * wave + fh;

    // The column's threshold and flip bit are fetched with the first operands, not after the K loop.
    const int col = col0 + fr;
    int thr = 0;
    uint32_t flip_word = 0u;
    if constexpr (FUSED) {
        thr = bn.thr[min(col, N - 1)];
        flip_word = bn.flip_bits[min(col, N - 1) >> 5];
    }

    // Two accumulators, so that consecutive MFMAs do not wait for each other's result.
    v16f acc[2];
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[0][v] = acc[1][v] = 0.0f;
    int ca = 0, cb = 0;

    // Quad indices are clamped into the row for the load and the quad zeroed afterwards, so the
    // loads of a batch carry no control flow and every lane runs every MFMA.
    uint4 qa[kBatch], qb[kBatch];
#pragma unroll
    for (int t = 0; t < kBatch; ++t) {
        const int q = min(first + kQuadStride * t, nq - 1);
        qa[t] = a_row[q];
        qb[t] = b_row[q];
    }
    for (int q0 = 0; q0 < nq; q0 += kQuadStride * kBatch) {
        uint4 na[kBatch], nb[kBatch];
        const int q1 = q0 + kQuadStride * kBatch;
        if (q1 < nq) {
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                const int q = min(q1 + first + kQuadStride * t, nq - 1);
                na[t] = a_row[q];
                nb[t] = b_row[q];
            }
        }
#pragma unroll
        for (int t = 0; t < kBatch; ++t) {
            const bool live = q0 + first + kQuadStride * t < nq;
            const uint4 a = zero_unless(live, qa[t]);
            const uint4 b = zero_unless(live, qb[t]);
            ca += popc4(a);
            cb += popc4(b);
#pragma unroll
            for (int s = 0; s < 4; ++s)
                acc[s & 1] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                    widen_fp4_a(quad_word(a, s)), widen_fp4_b(quad_word(b, s)), acc[s & 1], 4, 4, 0, 0, 0, 0);
        }
        if (q1 < nq) {
#pragma unroll
            for (int t = 0; t < kBatch; ++t) {
                qa[t] = na[t];
                qb[t] = nb[t];
            }
        }
    }

    // Lanes 0-31 end up with the popcount of A's row fr over both lane halves, lanes 32-63 with
    // that of B's row fr (one v_permlane32_swap exchanges the upper half of ca with the lower half of cb).
    const auto sw = __builtin_amdgcn_permlane32_swap(uint32_t(ca), uint32_t(cb), false, false);
    pop_part[wave][lane] = 2 * int(sw[0] + sw[1]);
#pragma unroll
    for (int g = 0; g < 4; ++g)
        part[wave][g][lane] = make_float4(acc[0][4 * g] + acc[1][4 * g], acc[0][4 * g + 1] + acc[1][4 * g + 1],
                                          acc[0][4 * g + 2] + acc[1][4 * g + 2], acc[0][4 * g + 3] + acc[1][4 * g + 3]);
    __syncthreads();

    // Accumulator register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32.  This wavefront
    // finishes registers 4*wave .. 4*wave + 3.
    float4 s4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    int4 pa4 = make_int4(0, 0, 0, 0);
    int pb = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
        const float4 p = part[w][wave][lane];
        s4.x += p.x; s4.y += p.y; s4.z += p.z; s4.w += p.w;
        const int4 pa = *reinterpret_cast<const int4*>(&pop_part[w][8 * wave + 4 * fh]);
        pa4.x += pa.x; pa4.y += pa.y; pa4.z += pa.z; pa4.w += pa.w;
        pb += pop_part[w][32 + fr];
    }
    const int base = K - pb;
    const int dot[4] = {base - pa4.x + (int(s4.x) << 2), base - pa4.y + (int(s4.y) << 2),
                        base - pa4.z + (int(s4.z) << 2), base - pa4.w + (int(s4.w) << 2)};
    if constexpr (!FUSED) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int row = row0 + 8 * wave + 4 * fh + e;
            if (row < M && col < N) C[int64_t(row) * ldc + col] = dot[e];
        }
    } else {
        const bool valid = col < N;
        const bool flip = (flip_word >> (col & 31)) & 1u;
        // Ballot e: low half = the word of row 8*wave + e, high half = that of row 8*wave + 4 + e.
        // Lane i < 8 stores row 8*wave + i.
        uint32_t word = 0u;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const uint64_t mask = __ballot(valid && ((dot[e] >= thr) != flip));
            if ((lane & 3) == e) word = (lane & 4) ? uint32_t(mask >> 32) : uint32_t(mask);
        }
        const int row = row0 + 8 * wave + lane;
        if (lane < 8 && row < M) bn.out[int64_t(row) * bn.ld_out + tn] = word;
    }
}

}  // namespace splitk

bool mfma_splitk_supports(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                          int64_t K) {
    return K >= 128 && K % 128 == 0 && K <= kMfmaMaxAcc && aligned_to(A, 16) && aligned_to(B, 16) && lda % 4 == 0 &&
           ldb % 4 == 0 && M >= 1 && N >= 1 && ceil_div(M, splitk::kTile) * ceil_div(N, splitk::kTile) <= kMaxDim;
}

// `bn.out == nullptr` selects the int32 form.  The caller has validated the arguments and
// checked mfma_splitk_supports.
int launch_xnor_gemm_mfma_splitk(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                                 int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, const BnSignArgs& bn,
                                 void* stream) {
    if (!mfma_splitk_supports(A, lda, B, ldb, M, N, K)) return BNN_ERR_UNSUPPORTED;
    const int tiles_m = int(ceil_div(M, splitk::kTile)), tiles_n = int(ceil_div(N, splitk::kTile));
    const dim3 grid(unsigned(int64_t(tiles_m) * tiles_n));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fused)
        hipLaunchKernelGGL((splitk::xnor_gemm_mfma_splitk_kernel<true>), grid, dim3(256), 0, s, A, lda, B, ldb,
                           static_cast<int32_t*>(nullptr), int64_t(0), int(M), int(N), int(K), tiles_m, tiles_n, bn);
    else
        hipLaunchKernelGGL((splitk::xnor_gemm_mfma_splitk_kernel<false>), grid, dim3(256), 0, s, A, lda, B, ldb, C, ldc,
                           int(M), int(N), int(K), tiles_m, tiles_n, bn);
    return check_launch();
}

}  // namespace bnn
