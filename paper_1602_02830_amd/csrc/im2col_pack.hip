// bnn_conv_im2col_pack: lowers a binary kh x kw convolution (3 x 3 in the
// paper's nets, Sec. 3.3) to the XNOR-popcount matrix product.
//
// Row m = (b*Ho + oy)*Wo + ox of the output is the receptive field of output
// pixel (b, oy, ox): K = kh*kw*Cin bits, bit (ky*kw + kx)*Cin + ci.  Taps
// outside the image are +1 (bit 1): zero padding seen through Eq. (1).
//
// HBM-bound on the write side: (kh*kw*Cin)/8 bytes written per output pixel;
// reads mostly hit cache (each input pixel is used kh*kw times).
//   quads   - Cin % 128 == 0 (the paper's layers): 16-byte copies.  A thread keeps one 16-byte unit
//             of the receptive field (its tap and channel quad, fixed for the kernel's life) and
//             walks over output pixels with carried (row, column) coordinates, so the copy loop
//             has no division; the threads of a pass write whole consecutive output rows.
//   words   - Cin % 32 == 0: every output word is a copy of one input word or all-ones.
//   bits    - any Cin: an output word gathers bit runs from up to 32 taps.
#include "bnn_internal.h"

namespace bnn {

struct ConvGeom {
    int B, H, W, Cin, Cw;        // Cw = words per input pixel
    int kh, kw, stride, pad;
    int Ho, Wo;
    int64_t M;                   // B*Ho*Wo
    int Kbits;                   // kh*kw*Cin
    int Kwords;                  // ceil(Kbits/32)
};

// VW = words moved per thread (1 or 4); Cin % (32*VW) == 0.
template <int VW>
__global__ __launch_bounds__(256) void im2col_words_kernel(const uint32_t* __restrict__ in, ConvGeom g,
                                                           uint32_t* __restrict__ out, int64_t ld_out,
                                                           int64_t n_units) {
    const int units_per_tap = g.Cw / VW;
    const int units_per_row = g.kh * g.kw * units_per_tap;
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < n_units;
         u += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = u / units_per_row;
        const int r = int(u - m * units_per_row);
        const int tap = r / units_per_tap;
        const int cu = r - tap * units_per_tap;
        const int ky = tap / g.kw, kx = tap - ky * g.kw;
        const int ox = int(m % g.Wo);
        const int64_t t = m / g.Wo;
        const int oy = int(t % g.Ho);
        const int64_t b = t / g.Ho;
        const int y = oy * g.stride + ky - g.pad;
        const int x = ox * g.stride + kx - g.pad;
        const bool inside = y >= 0 && y < g.H && x >= 0 && x < g.W;
        uint32_t* dst = out + m * ld_out + int64_t(tap) * g.Cw + cu * VW;
        const uint32_t* src = in + ((b * g.H + y) * g.W + x) * g.Cw + cu * VW;
        if (VW == 4) {
            uint4 v = make_uint4(~0u, ~0u, ~0u, ~0u);
            if (inside) v = *reinterpret_cast<const uint4*>(src);
            *reinterpret_cast<uint4*>(dst) = v;
        } else {
            *dst = inside ? *src : ~0u;
        }
    }
}

// Cin % 128 == 0, 16-byte aligned buffers, at most 256 units of 16 bytes per receptive field.
// Grid: (chunks of an image's output pixels, images).  P = 256 / units pixels per pass.
__global__ __launch_bounds__(256) void im2col_quads_kernel(const uint32_t* __restrict__ in, ConvGeom g,
                                                           uint32_t* __restrict__ out, int64_t ld_out,
                                                           int units, int pixels_per_block) {
    const int P = 256 / units;
    const int p = threadIdx.x / units, r = threadIdx.x - p * units;
    if (p >= P) return;                                  // 256 % units leftover threads
    const int units_per_tap = g.Cw / 4;
    const int tap = r / units_per_tap, cu = r - tap * units_per_tap;
    const int ky = tap / g.kw, kx = tap - ky * g.kw;
    const int n_pix = g.Ho * g.Wo;
    const int q_end = min((int(blockIdx.x) + 1) * pixels_per_block, n_pix);
    int q = int(blockIdx.x) * pixels_per_block + p;
    int oy = q / g.Wo, ox = q - oy * g.Wo;
    const int step_y = P / g.Wo, step_x = P - step_y * g.Wo;
    const int64_t b = blockIdx.y;
    const uint32_t* img = in + b * g.H * g.W * g.Cw + cu * 4;
    uint32_t* dst = out + (b * n_pix + q) * ld_out + tap * g.Cw + cu * 4;
    const int64_t dst_step = int64_t(P) * ld_out;
    for (; q < q_end; q += P) {
        const int y = oy * g.stride + ky - g.pad;
        const int x = ox * g.stride + kx - g.pad;
        uint4 v = make_uint4(~0u, ~0u, ~0u, ~0u);
        if (y >= 0 && y < g.H && x >= 0 && x < g.W)
            v = *reinterpret_cast<const uint4*>(img + (int64_t(y) * g.W + x) * g.Cw);
        *reinterpret_cast<uint4*>(dst) = v;
        dst += dst_step;
        ox += step_x;
        oy += step_y;
        if (ox >= g.Wo) {
            ox -= g.Wo;
            ++oy;
        }
    }
}

// `len` (1..32) bits of a pixel's channel vector starting at channel ci.
__device__ inline uint32_t channel_bits(const uint32_t* __restrict__ px, int ci, int len) {
    const int w = ci >> 5, s = ci & 31;
    uint32_t v = px[w] >> s;
    if (s + len > 32) v |= px[w + 1] << (32 - s);
    return len == 32 ? v : (v & ((1u << len) - 1u));
}

__global__ __launch_bounds__(256) void im2col_bits_kernel(const uint32_t* __restrict__ in, ConvGeom g,
                                                          uint32_t* __restrict__ out, int64_t ld_out,
                                                          int64_t n_units) {
    for (int64_t u = int64_t(blockIdx.x) * blockDim.x + threadIdx.x; u < n_units;
         u += int64_t(gridDim.x) * blockDim.x) {
        const int64_t m = u / g.Kwords;
        const int j = int(u - m * g.Kwords);
        const int ox = int(m % g.Wo);
        const int64_t t = m / g.Wo;
        const int oy = int(t % g.Ho);
        const int64_t b = t / g.Ho;
        const int k_end = min(32 * j + 32, g.Kbits);
        uint32_t word = 0u;
        int k = 32 * j;
        while (k < k_end) {
            const int tap = k / g.Cin;
            const int ci = k - tap * g.Cin;
            const int len = min(g.Cin - ci, k_end - k);
            const int ky = tap / g.kw, kx = tap - ky * g.kw;
            const int y = oy * g.stride + ky - g.pad;
            const int x = ox * g.stride + kx - g.pad;
            uint32_t bits = len == 32 ? ~0u : ((1u << len) - 1u);
            if (y >= 0 && y < g.H && x >= 0 && x < g.W)
                bits = channel_bits(in + ((b * g.H + y) * g.W + x) * g.Cw, ci, len);
            word |= bits << (k - 32 * j);
            k += len;
        }
        out[m * ld_out + j] = word;
    }
}

}  // namespace bnn

extern "C" int bnn_conv_im2col_pack(const uint32_t* in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                                    int kh, int kw, int stride, int pad, uint32_t* out, int64_t ld_out,
                                    void* stream) {
    using namespace bnn;
    if (B < 0 || H < 1 || W < 1 || Cin < 1 || kh < 1 || kw < 1 || stride < 1 || pad < 0)
        return BNN_ERR_INVALID_ARG;
    if (B > kMaxDim || H > kMaxDim || W > kMaxDim || Cin > kMaxDim) return BNN_ERR_INVALID_ARG;
    if (H + 2 * int64_t(pad) < kh || W + 2 * int64_t(pad) < kw) return BNN_ERR_INVALID_ARG;
    const int64_t Ho = (H + 2 * int64_t(pad) - kh) / stride + 1;
    const int64_t Wo = (W + 2 * int64_t(pad) - kw) / stride + 1;
    const int64_t kbits = int64_t(kh) * kw * Cin;
    if (kbits > kMaxK || Ho > kMaxDim || Wo > kMaxDim) return BNN_ERR_INVALID_ARG;
    const int64_t kwords = ceil_div(kbits, 32);
    if (ld_out < kwords) return BNN_ERR_INVALID_ARG;
    if (B == 0) return BNN_OK;
    if (!in || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(in, 4) || !aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;

    ConvGeom g;
    g.B = int(B); g.H = int(H); g.W = int(W); g.Cin = int(Cin); g.Cw = int(ceil_div(Cin, 32));
    g.kh = kh; g.kw = kw; g.stride = stride; g.pad = pad;
    g.Ho = int(Ho); g.Wo = int(Wo);
    g.M = B * Ho * Wo;
    g.Kbits = int(kbits); g.Kwords = int(kwords);

    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t max_blocks = 256 * 64;
    auto blocks_for = [&](int64_t units) {
        int64_t b = ceil_div(units, 256);
        return unsigned(b > max_blocks ? max_blocks : b);
    };
    if (Cin % 32 == 0) {
        const bool v4 = Cin % 128 == 0 && aligned_to(in, 16) && aligned_to(out, 16) && ld_out % 4 == 0;
        const int64_t row_units = kwords / 4, n_pix = Ho * Wo;
        if (v4 && row_units <= 256 && n_pix <= kMaxDim - 4096 && B <= 65535) {
            // Pixels per workgroup: a few passes each, and enough workgroups to fill the chip.
            const int P = int(256 / row_units);
            int64_t per_block = int64_t(P) * 8;
            while (per_block > P && ceil_div(n_pix, per_block) * B < 2048) per_block -= P;
            const dim3 grid(unsigned(ceil_div(n_pix, per_block)), unsigned(B));
            hipLaunchKernelGGL(im2col_quads_kernel, grid, dim3(256), 0, s, in, g, out, ld_out, int(row_units),
                               int(per_block));
        } else if (v4) {
            const int64_t units = g.M * (kwords / 4);
            hipLaunchKernelGGL(im2col_words_kernel<4>, dim3(blocks_for(units)), dim3(256), 0, s, in, g, out,
                               ld_out, units);
        } else {
            const int64_t units = g.M * kwords;
            hipLaunchKernelGGL(im2col_words_kernel<1>, dim3(blocks_for(units)), dim3(256), 0, s, in, g, out,
                               ld_out, units);
        }
    } else {
        const int64_t units = g.M * kwords;
        hipLaunchKernelGGL(im2col_bits_kernel, dim3(blocks_for(units)), dim3(256), 0, s, in, g, out, ld_out,
                           units);
    }
    return bnn::check_launch();
}
