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
// Used for every int32 output and for the fused output of the planes product.
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
    if constexpr (!FUSED) {
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
                        if (m < M && n < N) store_result(&C[int64_t(m) * ldc + n], dot);
                    }
                }
        }
    } else {
        // Fused epilogue of the planes product (the binary product has mfma_epilogue_bits below):
        //   bit(m, n) = (2S - rowsum >= thr[n]) XOR flip[n], i.e. S >= ceil((thr + rowsum) / 2).
        // A ballot over one accumulator register gives, in its low half, the 32-column word of
        // the row held by lanes 0-31 and, in its high half, that of the row 4 below.  The words
        // of one 32-row block are gathered with v_writelane so that lane r (block j = 0) and
        // lane 32 + r (block j = 1) end up holding row r's two words: one store per block row.
        static_assert(PLANES, "the binary product's fused epilogue is mfma_epilogue_bits");
        static_assert(WN == 2, "the fused epilogue pairs the two column blocks with the two lane halves");
        // While every term stays below 2^22 the comparison is done in float, where it is exact
        // (all terms are multiples of 1/2): S >= thr/2 + rowsum/2.  That is one add and one compare
        // per element instead of four integer operations.
        const bool fp_exact = 255 * int64_t(K) < (int64_t(1) << 22);
        int u1[WN];
        float tj[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int nl = wn * 32 * WN + j * 32 + fr;
            u1[j] = thr_s[nl] + 1;
            tj[j] = 0.5f * float(thr_s[nl]);
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
                            const bool p = FP ? (sacc >= tj[j] + pf) : (int(sacc) >= ((u1[j] + pa) >> 1));
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

// Largest K for which the fused binary epilogue below may fold its threshold into the accumulators:
// every term is a multiple of 1/8 and the largest magnitude is about 2K, exact in fp32 below 2^21.
constexpr int kMfmaFoldMaxK = 1 << 19;

// Column term of the folded threshold (see mfma_epilogue_bits): 1/8 - (thr - K + 2*popcount(B_n)) / 4,
// pop_b2 = 2*popcount(B_n), thr clamped to [-K-1, K+1].  Exact in fp32 for K <= kMfmaFoldMaxK.
__device__ inline float fold_column_term(int thr, int K, int pop_b2) {
    return 0.125f - 0.25f * float(thr - K + pop_b2);
}

// Fused epilogue (binary product) of a wavefront whose accumulators hold the TRANSPOSED blocks:
// the kernel issued its MFMAs with the operands swapped, so accumulator register v of lane l is
// column 8*(v/4) + 4*(l/32) + v%4 and row l%32 of its 32 x 32 block - a lane holds 16 columns of
// ONE output row, and the output bits of a row can be packed inside the lane, without ballots.
//
//   bit(m, n) = (K - 2pa - 2pb + 4S >= thr) XOR flip  =  (S - pa/2 - (thr - K + 2pb)/4 + 1/8 > 0) XOR flip
//
// (all terms multiples of 1/4, so adding 1/8 turns >= 0 into > 0 and the sum is never zero).
// For K <= kMfmaFoldMaxK the row term -pa/2 and the column term colfix_s[n] (fold_column_term)
// are added to all 1024 accumulators of a block by one v_mfma_f32_32x32x2_f32 (a rank-2 update:
// column term x 1 + 1 x row term, exact in fp32), after which the output bit is the complement of
// the accumulator's sign bit: one v_alignbit per accumulator shifts it into the lane's word.
// Larger K compare in integers.  The two lane halves hold alternate groups of 4 columns; one
// v_permlane32_swap brings the halves of column block 0 to lanes 0-31 and those of block 1 to
// lanes 32-63, so that, as in mfma_epilogue, lane l stores the word of column block l / 32.
// pop_a / pop_af / pop_b / thr_s / flip_s as in mfma_epilogue.
// mfma_output_words leaves, in words[i], the finished output word (flip and column validity
// applied) of tile row wm*32*WM + i*32 + fr and column block fh of this wavefront's column pair;
// mfma_epilogue_bits stores them.
template <int WM, int WN>
__device__ inline void mfma_output_words(v16f (&acc)[WM][WN], const int* pop_a, const float* pop_af,
                                         const int* pop_b, const int* thr_s, const uint32_t* flip_s,
                                         const float* colfix_s, int N, int K, int col0, int wm, int wn, int fr,
                                         int fh, uint32_t (&words)[WM]) {
    static_assert(WN == 2, "the two column blocks are paired with the two lane halves");
    const uint32_t flip_word = flip_s[wn * WN + fh];                    // col0 is a multiple of 32
    const int cols_left = N - (col0 + wn * 32 * WN + fh * 32);
    const uint32_t live_word = cols_left >= 32 ? ~0u : cols_left <= 0 ? 0u : ((1u << cols_left) - 1u);
    const bool fold = K <= kMfmaFoldMaxK;
    // Operands of the rank-2 update: lane (r, h) holds element [r][k = h] of the 32 x 2 left factor
    // (column term, 1) and element [k = h][r] of the 2 x 32 right factor (1, row term).
    float left[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) left[j] = fh == 0 ? colfix_s[wn * 32 * WN + j * 32 + fr] : 1.0f;
    if (fold) {
        // All rank-2 updates first: the vector-ALU work on a block then never waits for its own MFMA.
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            const float right = fh == 0 ? 1.0f : -pop_af[wm * 32 * WM + i * 32 + fr];
#pragma unroll
            for (int j = 0; j < WN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(left[j], right, acc[i][j], 0, 0, 0);
        }
    }
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int ml = wm * 32 * WM + i * 32 + fr;                       // this lane's row of the tile
        uint32_t part[WN];                                               // this lane's 16 columns: nibble g at bit 8g + 4*fh
        if (fold) {
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                // Sign bits of the block's 16 registers, nibble g (columns 8g + 4*fh ...) moved to bit 8g on the way.
                uint32_t neg = 0u;
#pragma unroll
                for (int g = 3; g >= 0; --g) {
#pragma unroll
                    for (int e = 3; e >= 0; --e)
                        neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[i][j][4 * g + e]), 31);
                    if (g > 0) neg <<= 4;
                }
                part[j] = (~neg & 0x0F0F0F0Fu) << (4 * fh);
            }
        } else {
            const int base_m = K - pop_a[ml];
#pragma unroll
            for (int j = 0; j < WN; ++j) {
                uint32_t bits = 0u;
#pragma unroll
                for (int g = 3; g >= 0; --g) {
                    const int nl = wn * 32 * WN + j * 32 + 8 * g + 4 * fh;
                    const int4 pb2 = *reinterpret_cast<const int4*>(&pop_b[nl]);
                    const int4 th = *reinterpret_cast<const int4*>(&thr_s[nl]);
#pragma unroll
                    for (int e = 3; e >= 0; --e) {
                        const int pb = e == 0 ? pb2.x : e == 1 ? pb2.y : e == 2 ? pb2.z : pb2.w;
                        const int t = e == 0 ? th.x : e == 1 ? th.y : e == 2 ? th.z : th.w;
                        const int dot = base_m - pb + (int(acc[i][j][4 * g + e]) << 2);
                        bits = (bits << 1) | (dot >= t ? 1u : 0u);
                    }
                }
                // Bit 4g + e of bits is column 8g + 4*fh + e of block j: move nibble g to bit 8g + 4*fh.
                uint32_t x = bits;
                x = (x | (x << 8)) & 0x00FF00FFu;
                x = (x | (x << 4)) & 0x0F0F0F0Fu;
                part[j] = x << (4 * fh);
            }
        }
        // Lanes 32-63 of part[0] <-> lanes 0-31 of part[1]: afterwards lane l holds, in the two
        // registers, the two halves of the word of column block l / 32.
        const auto sw = __builtin_amdgcn_permlane32_swap(part[0], part[1], false, false);
        words[i] = ((sw[0] | sw[1]) ^ flip_word) & live_word;
    }
}

template <int WM, int WN>
__device__ inline void mfma_epilogue_bits(v16f (&acc)[WM][WN], const int* pop_a, const float* pop_af,
                                          const int* pop_b, const int* thr_s, const uint32_t* flip_s,
                                          const float* colfix_s, const BnSignArgs& bn, int M, int N, int K,
                                          int row0, int col0, int wm, int wn, int fr, int fh) {
    uint32_t words[WM];
    mfma_output_words<WM, WN>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, colfix_s, N, K, col0, wm, wn, fr, fh, words);
    const int64_t nw = (int64_t(N) + 31) >> 5;
    const int64_t w = ((int64_t(col0) + wn * 32 * WN) >> 5) + fh;       // word column of this lane
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = row0 + wm * 32 * WM + i * 32 + fr;
        if (m < M && w < nw) bn.out[int64_t(m) * bn.ld_out + w] = words[i];
    }
}

}  // namespace bnn
