// Vector-ALU forms of the two products whose matrix-engine kernels stop at the exact range of fp32
// accumulation (sums below 2^24), so that the entry points keep working past it:
//
//   planes   a_1 = sum_{n=1..8} 2^(n-1) * <a_0^n, W^b_1>  (Alg. 4 step 1 / Sec. 1.6) for 255 * K >= 2^24
//   conv     the binary convolution of Sec. 3.3 as XnorDotProducts over receptive fields of more
//            than 2^24 bits
//
// Both are the paper's own formulation, Sec. 4 Eq. (5): per 32-bit word one logic operation and one
// population count, accumulated in integers, which is exact for any K the ABI admits.  With the
// pad bits masked, x in {0,1} and b in {0,1} standing for -1/+1:
//
//   planes:  sum_k x_k (2 b_k - 1) = 2 * popcount(x & b) - popcount(x)      per plane, weighted 2^p
//   conv:    sum_k (2a-1)(2b-1)    = K - 2 * popcount(a ^ b),  a = all ones for taps outside the image
//
// These kernels serve sizes far outside the paper's networks (more than 65 793 input features on
// the 8-bit first layer, receptive fields of more than 16.7 million bits); they are written to be
// correct and simple - one thread per output, a grid-stride loop - not fast.
#include "bnn_internal.h"
#include "gemm_staging.h"

namespace bnn {

template <bool FUSED>
__global__ __launch_bounds__(256) void bitplane_gemm_valu_kernel(const uint32_t* __restrict__ Xp, int64_t ldx,
                                                                 const uint32_t* __restrict__ B, int64_t ldb,
                                                                 int32_t* __restrict__ C, int64_t ldc, int M, int N,
                                                                 int K, BnSignArgs bn) {
    const int kw = (K + 31) >> 5;
    const uint32_t tmask = tail_mask(K);
    // FUSED: a thread owns one output WORD (32 columns of one row), else one output.
    const int64_t n_units = FUSED ? ((int64_t(N) + 31) >> 5) : int64_t(N);
    const int64_t total = int64_t(M) * n_units;
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < total; u += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = u / n_units, unit = u - m * n_units;
        const uint32_t* xrow = Xp + m * ldx;
        const int n0 = FUSED ? int(unit) * 32 : int(unit);
        const int cols = FUSED ? min(32, N - n0) : 1;
        uint32_t word = 0u;
        for (int c = 0; c < cols; ++c) {
            const uint32_t* brow = B + int64_t(n0 + c) * ldb;
            int32_t sum = 0;
            for (int w = 0; w < kw; ++w) {
                const uint32_t mask = w == kw - 1 ? tmask : ~0u;
                const uint32_t b = brow[w] & mask;
#pragma unroll
                for (int p = 0; p < 8; ++p) {
                    const uint32_t x = xrow[8 * w + p] & mask;
                    sum += (2 * __popc(x & b) - __popc(x)) * (1 << p);
                }
            }
            if (FUSED) word |= (sum >= bn.thr[n0 + c] ? 1u : 0u) << c;
            else C[m * ldc + n0] = sum;
        }
        if (FUSED) {
            const uint32_t live = cols >= 32 ? ~0u : ((1u << cols) - 1u);
            bn.out[m * bn.ld_out + unit] = (word ^ bn.flip_bits[unit]) & live;
        }
    }
}

template <bool FUSED>
__global__ __launch_bounds__(256) void conv_xnor_valu_kernel(const uint32_t* __restrict__ in,
                                                             const uint32_t* __restrict__ Wb, int64_t ldw,
                                                             int32_t* __restrict__ S, int64_t lds, int64_t M, int N,
                                                             int K, ConvArgs cv, BnSignArgs bn) {
    const int64_t n_units = FUSED ? ((int64_t(N) + 31) >> 5) : int64_t(N);
    const int64_t total = M * n_units;
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < total; u += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = u / n_units, unit = u - m * n_units;
        const int ox = int(m % cv.Wo);
        const int64_t t = m / cv.Wo;
        const int oy = int(t % cv.Ho);
        const int64_t b = t / cv.Ho;
        const uint32_t* img = in + b * cv.H * cv.W * cv.Cw;
        const int n0 = FUSED ? int(unit) * 32 : int(unit);
        const int cols = FUSED ? min(32, N - n0) : 1;
        uint32_t word = 0u;
        for (int c = 0; c < cols; ++c) {
            const uint32_t* frow = Wb + int64_t(n0 + c) * ldw;
            int32_t differ = 0;
            for (int ky = 0; ky < cv.kh; ++ky)
                for (int kx = 0; kx < cv.kw; ++kx) {
                    const int y = oy * cv.stride - cv.pad + ky, x = ox * cv.stride - cv.pad + kx;
                    const bool inside = y >= 0 && y < cv.H && x >= 0 && x < cv.W;
                    const uint32_t* px = img + (int64_t(inside ? y : 0) * cv.W + (inside ? x : 0)) * cv.Cw;
                    const uint32_t* fw = frow + int64_t(ky * cv.kw + kx) * cv.Cw;
                    for (int cw = 0; cw < cv.Cw; ++cw) differ += __popc((inside ? px[cw] : ~0u) ^ fw[cw]);
                }
            const int32_t dot = K - 2 * differ;
            if (FUSED) word |= (dot >= bn.thr[n0 + c] ? 1u : 0u) << c;
            else S[m * lds + n0] = dot;
        }
        if (FUSED) {
            const uint32_t live = cols >= 32 ? ~0u : ((1u << cols) - 1u);
            bn.out[m * bn.ld_out + unit] = (word ^ bn.flip_bits[unit]) & live;
        }
    }
}

static unsigned grid_for(int64_t total) {
    const int64_t blocks = ceil_div(total, 256);
    return unsigned(blocks < 1 ? 1 : (blocks > (int64_t(1) << 20) ? (int64_t(1) << 20) : blocks));
}

// The callers have validated the arguments.  fused: bn holds thresholds, flip words and the output.
int launch_bitplane_gemm_valu(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int32_t* C,
                              int64_t ldc, int64_t M, int64_t N, int64_t K, bool fused, BnSignArgs bn, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fused)
        hipLaunchKernelGGL(bitplane_gemm_valu_kernel<true>, dim3(grid_for(M * ceil_div(N, 32))), dim3(256), 0, s, Xp, ldx,
                           B, ldb, C, ldc, int(M), int(N), int(K), bn);
    else
        hipLaunchKernelGGL(bitplane_gemm_valu_kernel<false>, dim3(grid_for(M * N)), dim3(256), 0, s, Xp, ldx, B, ldb, C,
                           ldc, int(M), int(N), int(K), bn);
    return check_launch();
}

int launch_conv_xnor_valu(const uint32_t* in, const uint32_t* Wb, int64_t ldw, int32_t* S, int64_t lds, int64_t M,
                          int64_t N, int64_t K, ConvArgs cv, bool fused, BnSignArgs bn, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (fused)
        hipLaunchKernelGGL(conv_xnor_valu_kernel<true>, dim3(grid_for(M * ceil_div(N, 32))), dim3(256), 0, s, in, Wb, ldw, S,
                           lds, M, int(N), int(K), cv, bn);
    else
        hipLaunchKernelGGL(conv_xnor_valu_kernel<false>, dim3(grid_for(M * N)), dim3(256), 0, s, in, Wb, ldw, S, lds, M,
                           int(N), int(K), cv, bn);
    return check_launch();
}

}  // namespace bnn
