// Pieces shared by the packed-operand GEMM kernels: staging loads of packed
// rows, the die-aware tile order, and the arguments of the fused epilogue.
#pragma once

#include "bnn_internal.h"

namespace bnn {

// Loads words [4*quad, 4*quad+4) of row `row` (quad counted from the matrix's
// first word), zero where the row or word does not exist, pad bits masked.
template <bool VEC>
__device__ inline uint4 load_quad(const uint32_t* __restrict__ P, int64_t ld, int rows, int kw,
                                  uint32_t tmask, int row, int quad) {
    uint4 v = make_uint4(0u, 0u, 0u, 0u);
    const int w0 = quad * 4;
    if (row < rows && w0 < kw) {
        const uint32_t* p = P + int64_t(row) * ld + w0;
        if (VEC && w0 + 4 <= kw) {
            v = *reinterpret_cast<const uint4*>(p);
        } else {
            v.x = p[0];
            if (w0 + 1 < kw) v.y = p[1];
            if (w0 + 2 < kw) v.z = p[2];
            if (w0 + 3 < kw) v.w = p[3];
        }
        const int last = kw - 1 - w0;     // position of the row's last word inside this quad
        if (last == 0) v.x &= tmask;
        else if (last == 1) v.y &= tmask;
        else if (last == 2) v.z &= tmask;
        else if (last == 3) v.w &= tmask;
    }
    return v;
}

// Words [4*quad, 4*quad+4) of the row starting at `row_ptr`, with no checks: the caller
// guarantees the row exists and the quad is complete.  One 16-byte load when VEC.
template <bool VEC>
__device__ inline uint4 load_quad_unchecked(const uint32_t* __restrict__ row_ptr, int quad) {
    const uint32_t* p = row_ptr + quad * 4;
    if (VEC) return *reinterpret_cast<const uint4*>(p);
    return make_uint4(p[0], p[1], p[2], p[3]);
}

__device__ inline uint4 zero_unless(bool keep, uint4 v) {
    return make_uint4(keep ? v.x : 0u, keep ? v.y : 0u, keep ? v.z : 0u, keep ? v.w : 0u);
}

// Maps the hardware's round-robin placement of consecutive workgroups on the 8
// accelerator dies (each with its own L2) to compact panels of tiles: die d
// gets the contiguous range [d*per, (d+1)*per) of logical tile ids, and
// logical ids walk the tile grid in column-major bands of 8 tile-rows, so the
// tiles resident on one die at a time share a few A panels and B panels.
__device__ inline void tile_of_block(int bid, int tiles_m, int tiles_n, int& tm, int& tn) {
    const int total = tiles_m * tiles_n;
    constexpr int kDies = 8;
    int logical = bid;
    const int per = total / kDies;
    if (bid < per * kDies) logical = (bid % kDies) * per + bid / kDies;
    constexpr int kBand = 8;
    const int band_tiles = kBand * tiles_n;
    const int band = logical / band_tiles;
    const int in_band = logical - band * band_tiles;
    const int rows_in_band = min(kBand, tiles_m - band * kBand);
    tn = in_band / rows_in_band;
    tm = band * kBand + (in_band - tn * rows_in_band);
}

// Arguments of the fused epilogue (Alg. 4: a^b_k = Sign(BatchNorm(a_k, theta_k)) on folded
// thresholds), used when FUSED: the tile's pre-activations never leave registers.
struct BnSignArgs {
    const int32_t* thr;        // [N]
    const uint32_t* flip_bits; // [ceil(N/32)]
    uint32_t* out;             // [M][ld_out] packed bits
    int64_t ld_out;
};

// Geometry of a convolution whose receptive fields are gathered on the fly (implicit GEMM):
// input packed NHWC [B][H][W][Cw words], taps kh x kw, row m = (b*Ho + oy)*Wo + ox.
struct ConvArgs {
    int H, W, Cw, kh, kw, stride, pad, Ho, Wo;
};

}  // namespace bnn
