// Binary convolution layers without a materialised im2col matrix, and max pooling on bits.
//
// bnn_conv_xnor / bnn_conv_bn_sign_pack: a kh x kw binary convolution (3 x 3 in the paper's
// nets, Sec. 3.3) as the XnorDotProduct of Alg. 4 over receptive fields that the GEMM's tile
// loader gathers straight from the packed NHWC input (taps outside the image are +1: zero
// padding through Eq. (1)).  The kernels: the LDS-patch kernel (conv_patch.hip) for same-size
// convolutions whose tiles are whole image rows or images, else the conv modes of the matrix-engine
// GEMMs (xnor_gemm_mfma.hip, xnor_gemm_mfma_shortk.hip); launch_conv_mfma chooses.
//
// bnn_conv_pool_bn_sign_pack: the same layer with the paper's 2 x 2 max pooling between the
// convolution and BatchNorm + Sign, in one launch (LDS-patch kernel only).
//
// bnn_maxpool_bits: the paper's ConvNets pool the integer pre-activations before BatchNorm and
// Sign.  Sign(BatchNorm(.)) is monotone per channel - non-decreasing where the folded flip bit
// is 0, non-increasing where it is 1 - so Sign(BN(max over the window)) is the OR of the
// window's output bits where flip = 0 and their AND where flip = 1: pooling can run after the
// fused layer, on packed bits, 32 channels per operation.
#include "bnn_internal.h"
#include "gemm_staging.h"

namespace bnn {

bool mfma_path_supports(int64_t K);
int launch_conv_mfma(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                     int64_t N, int64_t K, ConvArgs cv, void* stream);
int launch_conv_mfma_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                           BnSignArgs bn, ConvArgs cv, void* stream);
int launch_conv_patch_pool_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                                 BnSignArgs bn, ConvArgs cv, void* stream);
// Vector-ALU form for receptive fields beyond the matrix engine's exact range (valu_fallbacks.hip).
int launch_conv_xnor_valu(const uint32_t* in, const uint32_t* Wb, int64_t ldw, int32_t* S, int64_t lds, int64_t M,
                          int64_t N, int64_t K, ConvArgs cv, bool fused, BnSignArgs bn, void* stream);

// Validates a convolution and fills the geometry.  M = B*Ho*Wo, K = kh*kw*Cin.
static int conv_geometry(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t Cin, const uint32_t* Wb,
                         int64_t ldw, int64_t Cout, int kh, int kw, int stride, int pad, ConvArgs& cv,
                         int64_t& M, int64_t& K) {
    if (B < 0 || H < 1 || W < 1 || Cin < 1 || Cout < 0 || kh < 1 || kw < 1 || stride < 1 || pad < 0)
        return BNN_ERR_INVALID_ARG;
    if (B > kMaxDim || H > 32767 || W > 32767 || Cin > kMaxDim || Cout > kMaxDim) return BNN_ERR_INVALID_ARG;
    if (H + 2 * int64_t(pad) < kh || W + 2 * int64_t(pad) < kw) return BNN_ERR_INVALID_ARG;
    const int64_t Ho = (H + 2 * int64_t(pad) - kh) / stride + 1;
    const int64_t Wo = (W + 2 * int64_t(pad) - kw) / stride + 1;
    // The tile loaders carry an output pixel as (oy << 16) | ox and form input coordinates in 32 bits.
    if (pad > 32767 || Ho > 32767 || Wo > 32767) return BNN_ERR_UNSUPPORTED;
    K = int64_t(kh) * kw * Cin;
    M = B * Ho * Wo;
    if (K > kMaxK || M > kMaxDim - 1024) return BNN_ERR_INVALID_ARG;      // row indices run up to one tile past M
    if (ldw < ceil_div(K, 32)) return BNN_ERR_INVALID_ARG;
    if (B > 0 && Cout > 0 && (!in || !Wb)) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(in, 4) || !aligned_to(Wb, 4)) return BNN_ERR_ALIGNMENT;
    // Whole channel words only.  With Cin % 128 == 0 the tile loaders move 16-byte groups of 4 channel
    // words; other multiples of 32 are taken word by word, by the LDS-patch kernel alone (same-size
    // stride-1 layers; launch_conv_mfma refuses the rest).  The input is addressed with 32-bit word offsets.
    if (Cin % 32 != 0) return BNN_ERR_UNSUPPORTED;
    if (Cin % 128 == 0 && !aligned_to(in, 16)) return BNN_ERR_UNSUPPORTED;
    if (B * H * W * (Cin / 32) > (int64_t(1) << 32) - 1) return BNN_ERR_UNSUPPORTED;
    cv.H = int(H); cv.W = int(W); cv.Cw = int(Cin / 32);
    cv.kh = kh; cv.kw = kw; cv.stride = stride; cv.pad = pad;
    cv.Ho = int(Ho); cv.Wo = int(Wo);
    return BNN_OK;
}

__global__ __launch_bounds__(256) void maxpool_bits_kernel(const uint32_t* __restrict__ in, int H, int W,
                                                           int Cw, int ph, int pw, int stride, int Hp, int Wp,
                                                           const uint32_t* __restrict__ flip_bits,
                                                           uint32_t* __restrict__ out, int64_t n_words) {
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < n_words;
         u += int64_t(gridDim.x) * blockDim.x) {
        const int cw = int(u % Cw);
        int64_t t = u / Cw;
        const int px = int(t % Wp);
        t /= Wp;
        const int py = int(t % Hp);
        const int64_t b = t / Hp;
        uint32_t any = 0u, all = ~0u;
        for (int dy = 0; dy < ph; ++dy)
            for (int dx = 0; dx < pw; ++dx) {
                const uint32_t v = in[((b * H + py * stride + dy) * W + px * stride + dx) * Cw + cw];
                any |= v;
                all &= v;
            }
        const uint32_t flip = flip_bits ? flip_bits[cw] : 0u;
        out[u] = (any & ~flip) | (all & flip);
    }
}

}  // namespace bnn

extern "C" int bnn_conv_xnor(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t Cin, const uint32_t* Wb,
                             int64_t ldw, int64_t Cout, int kh, int kw, int stride, int pad, int32_t* S,
                             int64_t lds, void* stream) {
    using namespace bnn;
    ConvArgs cv;
    int64_t M, K;
    const int st = conv_geometry(in, B, H, W, Cin, Wb, ldw, Cout, kh, kw, stride, pad, cv, M, K);
    if (st != BNN_OK) return st;
    if (lds < Cout) return BNN_ERR_INVALID_ARG;
    if (M == 0 || Cout == 0) return BNN_OK;
    if (!S) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(S, 4)) return BNN_ERR_ALIGNMENT;
    if (!mfma_path_supports(K)) return launch_conv_xnor_valu(in, Wb, ldw, S, lds, M, Cout, K, cv, false, BnSignArgs{}, stream);
    return launch_conv_mfma(in, Wb, ldw, S, lds, M, Cout, K, cv, stream);
}

extern "C" int bnn_conv_bn_sign_pack(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                                     const uint32_t* Wb, int64_t ldw, int64_t Cout, int kh, int kw, int stride,
                                     int pad, const int32_t* thr, const uint32_t* flip_bits, uint32_t* out,
                                     int64_t ld_out, void* stream) {
    using namespace bnn;
    ConvArgs cv;
    int64_t M, K;
    const int st = conv_geometry(in, B, H, W, Cin, Wb, ldw, Cout, kh, kw, stride, pad, cv, M, K);
    if (st != BNN_OK) return st;
    if (ld_out < ceil_div(Cout, 32)) return BNN_ERR_INVALID_ARG;
    if (M == 0 || Cout == 0) return BNN_OK;
    if (!thr || !flip_bits || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(thr, 4) || !aligned_to(flip_bits, 4) || !aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;
    if (!mfma_path_supports(K))
        return launch_conv_xnor_valu(in, Wb, ldw, nullptr, 0, M, Cout, K, cv, true, BnSignArgs{thr, flip_bits, out, ld_out},
                                     stream);
    return launch_conv_mfma_fused(in, Wb, ldw, M, Cout, K, BnSignArgs{thr, flip_bits, out, ld_out}, cv, stream);
}

extern "C" int bnn_conv_pool_bn_sign_pack(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                                          const uint32_t* Wb, int64_t ldw, int64_t Cout, int kh, int kw, int stride,
                                          int pad, int pool, const int32_t* thr, const uint32_t* flip_bits,
                                          uint32_t* out, int64_t ld_out, void* stream) {
    using namespace bnn;
    ConvArgs cv;
    int64_t M, K;
    const int st = conv_geometry(in, B, H, W, Cin, Wb, ldw, Cout, kh, kw, stride, pad, cv, M, K);
    if (st != BNN_OK) return st;
    if (pool < 1 || ld_out < ceil_div(Cout, 32)) return BNN_ERR_INVALID_ARG;
    if (pool != 2 || !mfma_path_supports(K)) return BNN_ERR_UNSUPPORTED;
    if (M == 0 || Cout == 0) return BNN_OK;
    if (!thr || !flip_bits || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(thr, 4) || !aligned_to(flip_bits, 4) || !aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;
    return launch_conv_patch_pool_fused(in, Wb, ldw, M, Cout, K, BnSignArgs{thr, flip_bits, out, ld_out}, cv, stream);
}

extern "C" int bnn_maxpool_bits(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t C, int ph, int pw,
                                int stride, const uint32_t* flip_bits, uint32_t* out, void* stream) {
    using namespace bnn;
    if (B < 0 || H < 1 || W < 1 || C < 1 || ph < 1 || pw < 1 || stride < 1) return BNN_ERR_INVALID_ARG;
    if (B > kMaxDim || H > kMaxDim || W > kMaxDim || C > kMaxDim || H < ph || W < pw) return BNN_ERR_INVALID_ARG;
    if (B == 0) return BNN_OK;
    if (!in || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(in, 4) || !aligned_to(out, 4) || !aligned_to(flip_bits, 4)) return BNN_ERR_ALIGNMENT;
    const int64_t Hp = (H - ph) / stride + 1, Wp = (W - pw) / stride + 1;
    const int64_t Cw = ceil_div(C, 32);
    const int64_t n_words = B * Hp * Wp * Cw;
    int64_t blocks = ceil_div(n_words, 256);
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(maxpool_bits_kernel, dim3(unsigned(blocks)), dim3(256), 0, static_cast<hipStream_t>(stream),
                       in, int(H), int(W), int(Cw), ph, pw, stride, int(Hp), int(Wp), flip_bits, out, n_words);
    return check_launch();
}
