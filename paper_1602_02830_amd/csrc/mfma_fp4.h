// Pieces shared by the matrix-engine (fp4 MFMA) kernels: bit widening, row sums, and the
// epilogue that turns the MFMA sums into +-1 dot products or packed output bits.
#pragma once

#include <type_traits>

#include "bnn_internal.h"
#include "gemm_staging.h"

namespace bnn {

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kMfmaKT = 16;              // words of A per row and staged tile
constexpr int kMfmaKQ = kMfmaKT / 4;     // 16-byte quads per row per tile
constexpr int64_t kMfmaMaxAcc = int64_t(1) << 24;   // exact fp32 accumulation of non-negative integers

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

// Sum over k of the four plane words of a quad weighted 2^p0 .. 2^(p0+3).
__device__ inline int popc4_weighted(uint4 v, int p0) {
    return (__popc(v.x) + 2 * __popc(v.y) + 4 * __popc(v.z) + 8 * __popc(v.w)) << p0;
}

__device__ inline uint32_t quad_word(const uint4& q, int s) { return s == 0 ? q.x : s == 1 ? q.y : s == 2 ? q.z : q.w; }

// Epilogue of a wavefront that owns WM x WN blocks of 32 x 32 fp32 accumulators at block
// position (wm, wn) of a (64*WM) x (64*WN) workgroup tile whose first row / column is row0 / col0.
// pop_a[tile row] / pop_b[tile column] hold 2*popcount (binary) or the plain row sum of the 8-bit
// inputs (planes, pop_b unused); pop_af[tile row] = pop_a / 4 (binary) or / 2 (planes) as float;
// thr_s[tile column] / flip_s[tile column / 32]: the tile's thresholds and flip words (fused only,
// zero for columns beyond N).
// fr = lane % 32, fh = lane / 32.
template <int WM, int WN, bool FUSED, bool PLANES>
__device__ inline void mfma_epilogue(const v16f (&acc)[WM][WN], const int* pop_a, const float* pop_af,
                                     const int* pop_b, const int* thr_s, const uint32_t* flip_s,
                                     int32_t* __restrict__ C, int64_t ldc, const BnSignArgs& bn, int M, int N, int K,
                                     int row0, int col0, int wm, int wn, int fr, int fh) {
    // Result from the matrix-engine sum S:  binary  K - 2pa - 2pb + 4S,   planes  2S - rowsum.
    // Accumulator register v of lane l: row 8*(v/4) + 4*(l/32) + v%4, column l%32 of its 32x32 block.
    constexpr int kShift = PLANES ? 1 : 2;
    if (!FUSED) {
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int nl = wn * 32 * WN + j * 32 + fr;
            const int n = col0 + nl;
            const int base_n = PLANES ? 0 : K - pop_b[nl];
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
                        const int dot = base_n - pa + (int(acc[i][j][4 * vq + e]) << kShift);
                        if (m < M && n < N) __builtin_nontemporal_store(dot, &C[int64_t(m) * ldc + n]);
                    }
                }
        }
    } else {
        // bit(m, n) = (result >= thr[n]) XOR flip[n], i.e.
        //   binary: S >= ceil((thr - K + 2pb + 2pa) / 4),   planes: S >= ceil((thr + rowsum) / 2).
        // A ballot over one accumulator register gives, in its low half, the 32-column word of
        // the row held by lanes 0-31 and, in its high half, that of the row 4 below.  The words
        // of one 32-row block are gathered with v_writelane so that lane r (block j = 0) and
        // lane 32 + r (block j = 1) end up holding row r's two words: one store per block row.
        static_assert(WN == 2, "the fused epilogue pairs the two column blocks with the two lane halves");
        // While every term stays below 2^22 the comparison is done in float, where it is exact
        // (all terms are multiples of 1/4): S >= (thr - K + 2pb)/4 + 2pa/4, resp. S >= thr/2 + rowsum/2.
        // That is one add and one compare per element instead of four integer operations.
        const bool fp_exact = PLANES ? (255 * int64_t(K) < (int64_t(1) << 22)) : (K <= (1 << 21));
        int u3[WN];
        float tj[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int nl = wn * 32 * WN + j * 32 + fr;
            const int cj = PLANES ? thr_s[nl] : thr_s[nl] - K + pop_b[nl];
            u3[j] = cj + (PLANES ? 1 : 3);
            tj[j] = (PLANES ? 0.5f : 0.25f) * float(cj);
        }
        // Flip and validity are applied to whole output words after the gather: lane l holds the
        // word of column block l / 32, whose flip word is flip_s[...] and whose valid bits are the
        // columns below N.
        const int64_t nw = (int64_t(N) + 31) >> 5;
        const int64_t w = ((int64_t(col0) + wn * 32 * WN) >> 5) + fh;       // word column of this lane
        const uint32_t flip_word = flip_s[wn * WN + fh];                    // col0 is a multiple of 32
        const int cols_left = N - (col0 + wn * 32 * WN + fh * 32);
        const uint32_t live_word = cols_left >= 32 ? ~0u : cols_left <= 0 ? 0u : ((1u << cols_left) - 1u);
        auto pack_and_store = [&](auto fp_tag) {
            constexpr bool FP = decltype(fp_tag)::value;
#pragma unroll
            for (int i = 0; i < WM; ++i) {
                int words = 0;
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const int ml = wm * 32 * WM + i * 32 + 8 * vq + 4 * fh;
                    const int4 pa2 = *reinterpret_cast<const int4*>(&pop_a[ml]);
                    const float4 paf = *reinterpret_cast<const float4*>(&pop_af[ml]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int pa = e == 0 ? pa2.x : e == 1 ? pa2.y : e == 2 ? pa2.z : pa2.w;
                        const float pf = e == 0 ? paf.x : e == 1 ? paf.y : e == 2 ? paf.z : paf.w;
#pragma unroll
                        for (int j = 0; j < WN; ++j) {
                            const float sacc = acc[i][j][4 * vq + e];
                            const bool p = FP ? (sacc >= tj[j] + pf) : (int(sacc) >= ((u3[j] + pa) >> kShift));
                            const uint64_t mask = __ballot(p);
                            words = bnn_llvm_writelane(int(uint32_t(mask)), 32 * j + 8 * vq + e, words);
                            words = bnn_llvm_writelane(int(uint32_t(mask >> 32)), 32 * j + 8 * vq + 4 + e, words);
                        }
                    }
                }
                const int m = row0 + wm * 32 * WM + i * 32 + fr;
                if (m < M && w < nw) bn.out[int64_t(m) * bn.ld_out + w] = (uint32_t(words) ^ flip_word) & live_word;
            }
        };
        if (fp_exact) pack_and_store(std::true_type{});
        else pack_and_store(std::false_type{});
    }
}

}  // namespace bnn
