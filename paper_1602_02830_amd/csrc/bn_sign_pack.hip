// bnn_bn_sign_pack: a^b_k = Sign(BatchNorm(a_k, theta_k)) of Alg. 4 on folded
// per-channel integer thresholds, written as packed bits for the next layer.
//
//   out[m][n/32] bit (n%32) = (C[m][n] >= thr[n]) XOR flip[n]
//
// HBM-bound streaming kernel (4 B read, 1/8 B written per element; thresholds
// and flip words stay in cache).  Same work split as the Sign packer: an
// aligned group of 8 lanes produces one output word, each lane comparing 4
// consecutive int32 (one 16-byte load on the fast path), nibbles combined by
// three DPP permutes.  Rows that are whole numbers of 128 channels take
// bn_sign_pack_units_kernel (4 words per group, thresholds in registers,
// 16-byte stores); everything else bn_sign_pack_kernel.
#include "bnn_internal.h"

namespace bnn {

// 16-byte load of pre-activations.  ONCE: non-temporal, for matrices larger than the last-level cache (1 GiB:
// 5.94 -> 6.01 TB/s); smaller ones are usually still cached from the product that wrote them, where a
// non-temporal read does not find them (164 MB: 5.8 -> 5.0 TB/s).  The thresholds, read by every row, always
// keep the default policy.
constexpr int64_t kOnceMinBytes = int64_t(256) << 20;
template <bool ONCE>
__device__ inline int4 load_preact(const int32_t* p) {
    if (!ONCE) return *reinterpret_cast<const int4*>(p);
    typedef int i4 __attribute__((ext_vector_type(4)));
    const i4 t = __builtin_nontemporal_load(reinterpret_cast<const i4*>(p));
    return make_int4(t[0], t[1], t[2], t[3]);
}

constexpr int kBnThreads = 256;
constexpr int kBnUnroll = 4;
// Rows a workgroup of the fast path walks down with its thresholds in registers.  Measured on a 1 GiB input:
// 1 row 5.83 TB/s, 2 rows 5.95, 4 rows 5.75, 8 rows 5.60 (with or without the next row's loads issued early):
// short-lived workgroups keep the addresses in flight close together, which matters more than the saved
// threshold loads.
constexpr int kBnUnitSteps = 2;

template <bool VEC, bool ONCE>
__global__ __launch_bounds__(kBnThreads) void bn_sign_pack_kernel(
    const int32_t* __restrict__ C, int64_t ldc, int64_t M, int64_t N,
    const int32_t* __restrict__ thr, const uint32_t* __restrict__ flip_bits,
    uint32_t* __restrict__ out, int64_t ld_out, int64_t nw, int64_t n_words, int64_t slice_row, int64_t slice_word,
    int64_t pass_row, int64_t pass_word) {
    // Word groups are numbered row-major (g = row * nw + word).  A workgroup takes kBnUnroll consecutive
    // slices of 32 groups per pass (16 KB of contiguous input when rows are dense), thread t group t/8 of
    // each slice; passes are a whole grid apart.  (row, word) are stepped by (groups / nw, groups % nw)
    // with a carry: one division per thread, not per group.
    constexpr int kSlice = kBnThreads / 8;
    const int q = threadIdx.x & 7;
    const int64_t pass_groups = int64_t(gridDim.x) * kSlice * kBnUnroll;
    int64_t g0 = int64_t(blockIdx.x) * kSlice * kBnUnroll + (threadIdx.x >> 3);
    int64_t row0 = g0 / nw, w0 = g0 - row0 * nw;

    for (; g0 < n_words; g0 += pass_groups) {
        int4 c[kBnUnroll], t[kBnUnroll];
        int64_t row_of[kBnUnroll], word_of[kBnUnroll];
        int64_t row = row0, w = w0;
        if (VEC && N >= 4) {
            // Unconditional 16-byte loads of the pre-activations and of their thresholds, all in flight
            // together: a lane whose four channels do not all exist (a slice past the last group, the tail
            // of a row) loads the row's last whole quad of channels instead - an address inside the matrix -
            // and what it needs is sorted out afterwards.
            const int64_t n_last = (N & ~int64_t(3)) - 4;
            bool whole[kBnUnroll];
#pragma unroll
            for (int u = 0; u < kBnUnroll; ++u) {
                const bool live = g0 + u * kSlice < n_words;
                row_of[u] = live ? row : -1;
                word_of[u] = w;
                const int64_t n0 = w * 32 + q * 4;
                whole[u] = live && n0 + 3 < N;
                const int64_t n_at = whole[u] ? n0 : n_last;
                c[u] = load_preact<ONCE>(C + (live ? row : 0) * ldc + n_at);
                t[u] = *reinterpret_cast<const int4*>(thr + n_at);
                row += slice_row;
                w += slice_word;
                if (w >= nw) {
                    w -= nw;
                    ++row;
                }
            }
#pragma unroll
            for (int u = 0; u < kBnUnroll; ++u) {
                const int64_t n0 = word_of[u] * 32 + q * 4;
                if (!whole[u]) {
                    c[u] = make_int4(0, 0, 0, 0);
                    t[u] = make_int4(0, 0, 0, 0);
                    if (row_of[u] >= 0 && n0 < N) {                    // a row's last, partial quad (N % 4 != 0)
                        const int32_t* p = C + row_of[u] * ldc + n0;
                        if (n0 + 0 < N) { c[u].x = p[0]; t[u].x = thr[n0 + 0]; }
                        if (n0 + 1 < N) { c[u].y = p[1]; t[u].y = thr[n0 + 1]; }
                        if (n0 + 2 < N) { c[u].z = p[2]; t[u].z = thr[n0 + 2]; }
                    }
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < kBnUnroll; ++u) {
                const bool live = g0 + u * kSlice < n_words;
                row_of[u] = live ? row : -1;
                word_of[u] = w;
                const int64_t n0 = w * 32 + q * 4;
                const int32_t* p = C + row * ldc + n0;
                c[u] = make_int4(0, 0, 0, 0);
                t[u] = make_int4(0, 0, 0, 0);
                if (live) {
                    if (n0 + 0 < N) { c[u].x = p[0]; t[u].x = thr[n0 + 0]; }
                    if (n0 + 1 < N) { c[u].y = p[1]; t[u].y = thr[n0 + 1]; }
                    if (n0 + 2 < N) { c[u].z = p[2]; t[u].z = thr[n0 + 2]; }
                    if (n0 + 3 < N) { c[u].w = p[3]; t[u].w = thr[n0 + 3]; }
                }
                row += slice_row;
                w += slice_word;
                if (w >= nw) {
                    w -= nw;
                    ++row;
                }
            }
        }
        row0 += pass_row;
        w0 += pass_word;
        if (w0 >= nw) {
            w0 -= nw;
            ++row0;
        }
#pragma unroll
        for (int u = 0; u < kBnUnroll; ++u) {
            const int64_t n0 = word_of[u] * 32 + q * 4;
            // Bits of channels >= N: flip word has zero pad bits, and the mask below clears them.
            const uint32_t flip = (flip_bits[word_of[u]] >> (4 * q)) & 0xFu;
            uint32_t nib = uint32_t(c[u].x >= t[u].x) | (uint32_t(c[u].y >= t[u].y) << 1) |
                           (uint32_t(c[u].z >= t[u].z) << 2) | (uint32_t(c[u].w >= t[u].w) << 3);
            nib ^= flip;
            const int64_t valid = N - n0;                       // channels left from this lane's first
            const uint32_t vmask = valid >= 4 ? 0xFu : (valid <= 0 ? 0u : ((1u << valid) - 1u));
            nib &= vmask;
            const uint32_t word = or_reduce8(nib << (4 * q));
            if (q == 0 && row_of[u] >= 0) out[row_of[u] * ld_out + word_of[u]] = word;
        }
    }
}

// Fast path for rows that are whole numbers of 128-channel units (see UnitSplit).  A workgroup walks down
// `steps` consecutive rows on the same columns, so a lane's 16 thresholds and flip nibbles are loaded
// once and stay in registers: per 16 bytes of pre-activations there is no second (cached) 16-byte
// threshold load and no flip-word load.  Lane 0 of a group writes its 4 output words with one
// 16-byte store.
template <bool ONCE>
__global__ __launch_bounds__(kBnThreads) void bn_sign_pack_units_kernel(
    const int32_t* __restrict__ C, int64_t ldc, int64_t M, const int32_t* __restrict__ thr,
    const uint32_t* __restrict__ flip_bits, uint32_t* __restrict__ out, int64_t ld_out, UnitSplit us) {
    const int q = threadIdx.x & 7, gi = threadIdx.x >> 3;
    const int64_t block_row = int64_t(blockIdx.x) / us.slices_per_row;
    const int slice = int(int64_t(blockIdx.x) - block_row * us.slices_per_row);
    const int unit = us.rows_per_step == 1 ? slice * 32 + gi : gi % us.units_per_row;
    const int row_in_step = us.rows_per_step == 1 ? 0 : gi / us.units_per_row;
    const int64_t n0 = int64_t(unit) * 128 + q * 4;
    int4 t[4];
    uint32_t flip[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        t[u] = *reinterpret_cast<const int4*>(thr + n0 + 32 * u);
        flip[u] = (flip_bits[int64_t(unit) * 4 + u] >> (4 * q)) & 0xFu;
    }
    for (int i = 0; i < us.steps; ++i) {
        const int64_t row = (block_row * us.steps + i) * us.rows_per_step + row_in_step;
        if (row >= M) break;
        const int32_t* p = C + row * ldc + n0;
        int4 c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = load_preact<ONCE>(p + 32 * u);
        uint32_t w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t nib = (uint32_t(c[u].x >= t[u].x) | (uint32_t(c[u].y >= t[u].y) << 1) |
                                  (uint32_t(c[u].z >= t[u].z) << 2) | (uint32_t(c[u].w >= t[u].w) << 3)) ^ flip[u];
            w[u] = or_reduce8(nib << (4 * q));
        }
        if (q == 0) *reinterpret_cast<uint4*>(out + row * ld_out + int64_t(unit) * 4) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

}  // namespace bnn

extern "C" int bnn_bn_sign_pack(const int32_t* C, int64_t ldc, int64_t M, int64_t N,
                                const int32_t* thr, const uint32_t* flip_bits, uint32_t* out,
                                int64_t ld_out, void* stream) {
    using namespace bnn;
    if (M < 0 || N < 0 || M > kMaxDim || N > kMaxDim) return BNN_ERR_INVALID_ARG;
    const int64_t nw = ceil_div(N, 32);
    if (ldc < N || ld_out < nw) return BNN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return BNN_OK;
    if (!C || !thr || !flip_bits || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(C, 4) || !aligned_to(thr, 4) || !aligned_to(flip_bits, 4) || !aligned_to(out, 4))
        return BNN_ERR_ALIGNMENT;

    const int64_t n_words = M * nw;
    int64_t blocks = ceil_div(n_words, int64_t(kBnThreads / 8) * kBnUnroll);
    const int64_t max_blocks = int64_t(1) << 20;   // one pass per workgroup up to 16 GiB of input
    if (blocks > max_blocks) blocks = max_blocks;
    const bool vec = aligned_to(C, 16) && aligned_to(thr, 16) && ldc % 4 == 0;
    const bool once = M * N * int64_t(sizeof(int32_t)) > kOnceMinBytes;          // see load_preact
    const int64_t slice = kBnThreads / 8, pass = blocks * slice * kBnUnroll;
    hipStream_t s = static_cast<hipStream_t>(stream);
    UnitSplit us;
    if (vec && aligned_to(out, 16) && ld_out % 4 == 0 && unit_split(N, kBnUnitSteps, us)) {
        const int64_t unit_blocks = ceil_div(M, int64_t(us.rows_per_step) * us.steps) * us.slices_per_row;
        if (unit_blocks <= kMaxDim) {
            if (once)
                hipLaunchKernelGGL(bn_sign_pack_units_kernel<true>, dim3(unsigned(unit_blocks)), dim3(kBnThreads), 0, s, C, ldc, M,
                                   thr, flip_bits, out, ld_out, us);
            else
                hipLaunchKernelGGL(bn_sign_pack_units_kernel<false>, dim3(unsigned(unit_blocks)), dim3(kBnThreads), 0, s, C, ldc, M,
                                   thr, flip_bits, out, ld_out, us);
            return check_launch();
        }
    }
    if (vec && once)
        hipLaunchKernelGGL((bn_sign_pack_kernel<true, true>), dim3(unsigned(blocks)), dim3(kBnThreads), 0, s, C, ldc,
                           M, N, thr, flip_bits, out, ld_out, nw, n_words, slice / nw, slice % nw, pass / nw, pass % nw);
    else if (vec)
        hipLaunchKernelGGL((bn_sign_pack_kernel<true, false>), dim3(unsigned(blocks)), dim3(kBnThreads), 0, s, C, ldc,
                           M, N, thr, flip_bits, out, ld_out, nw, n_words, slice / nw, slice % nw, pass / nw, pass % nw);
    else
        hipLaunchKernelGGL((bn_sign_pack_kernel<false, false>), dim3(unsigned(blocks)), dim3(kBnThreads), 0, s, C, ldc,
                           M, N, thr, flip_bits, out, ld_out, nw, n_words, slice / nw, slice % nw, pass / nw, pass % nw);
    return check_launch();
}
