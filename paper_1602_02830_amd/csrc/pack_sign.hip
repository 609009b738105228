// bnn_pack_sign: Eq. (1) binarisation fused with the 32-per-word packing of Sec. 4.
//
// HBM-bound streaming kernel: 4 B read and 1/8 B written per element.
// Work unit: one output word = 32 consecutive elements of a row, handled by an
// aligned group of 8 lanes; each lane reads 4 consecutive floats (one 16-byte
// load on the fast path), forms a 4-bit nibble and the group ORs the shifted
// nibbles together with three DPP permutes.  A wavefront therefore reads eight
// 128-byte segments and writes eight words per step, and groups never straddle
// a row, so rows whose length is not a multiple of 32 cost nothing extra apart
// from their own partial last word.  Rows that are whole numbers of 128 elements
// take pack_sign_units_kernel (4 words per group, one 16-byte store).
#include "bnn_internal.h"

namespace bnn {

constexpr int kPackThreads = 256;
constexpr int kPackUnroll = 4;   // words per group of 8 lanes per pass (loads in flight)

__device__ inline uint32_t ge_zero(float v) { return v >= 0.0f ? 1u : 0u; }

// 16-byte load of the input.  ONCE: non-temporal, for inputs larger than the last-level cache, where nothing
// read now is found again later and the default policy only displaces what else is cached (1 GiB input:
// 6.02 -> 6.45 TB/s).  Inputs that fit the cache keep the default policy: they are often still there from
// their producer or from the previous step, and a non-temporal read does not find them (31 MB MLP input,
// re-read every step: 5.8 -> 5.5 TB/s non-temporally).
constexpr int64_t kOnceMinBytes = int64_t(256) << 20;
template <bool ONCE>
__device__ inline float4 load_input(const float* p) {
    if (!ONCE) return *reinterpret_cast<const float4*>(p);
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 t = __builtin_nontemporal_load(reinterpret_cast<const f4*>(p));
    return make_float4(t[0], t[1], t[2], t[3]);
}

// Word groups are numbered row-major (g = row * kw + word).  (row, word) coordinates are stepped by a
// constant number of groups with a carry instead of being divided out for every group.
struct WordStep {
    int64_t d_row;   // groups / kw
    int64_t d_word;  // groups % kw
};

inline WordStep word_step(int64_t groups, int64_t kw) { return WordStep{groups / kw, groups % kw}; }

__device__ inline void advance(int64_t& row, int64_t& w, const WordStep& st, int64_t kw) {
    row += st.d_row;
    w += st.d_word;
    if (w >= kw) {
        w -= kw;
        ++row;
    }
}

// A workgroup takes kPackUnroll consecutive slices of 32 word groups per pass (16 KB of contiguous
// input when rows are dense), thread t group t/8 of each slice; passes are a whole grid apart.
template <bool VEC, bool ONCE>
__global__ __launch_bounds__(kPackThreads) void pack_sign_kernel(
    const float* __restrict__ x, int64_t rows, int64_t cols, int64_t ld_x,
    uint32_t* __restrict__ out, int64_t ld_out, int64_t kw, int64_t n_words, WordStep slice, WordStep pass) {
    constexpr int kSlice = kPackThreads / 8;             // word groups per slice
    const int q = threadIdx.x & 7;                       // lane within its group
    const int64_t pass_groups = int64_t(gridDim.x) * kSlice * kPackUnroll;
    int64_t g0 = int64_t(blockIdx.x) * kSlice * kPackUnroll + (threadIdx.x >> 3);
    int64_t row0 = g0 / kw, w0 = g0 - row0 * kw;         // the only division of the thread

    for (; g0 < n_words; g0 += pass_groups) {
        float v[kPackUnroll][4];
        int64_t word_of[kPackUnroll];
        int64_t row_of[kPackUnroll];
        int64_t row = row0, w = w0;
        if (VEC && cols >= 4) {
            // Four unconditional 16-byte loads, all in flight together: a lane whose four elements do not all
            // exist (a slice past the last group, the tail of a row) loads the row's last whole quad of
            // elements instead - an address inside the matrix - and what it needs is sorted out afterwards.
            const int64_t c_last = (cols & ~int64_t(3)) - 4;         // first element of that quad (16-byte aligned)
            float4 f[kPackUnroll];
            bool whole[kPackUnroll];
            int64_t c_of[kPackUnroll];
#pragma unroll
            for (int u = 0; u < kPackUnroll; ++u) {
                const bool live = g0 + u * kSlice < n_words;
                row_of[u] = live ? row : -1;
                word_of[u] = w;
                c_of[u] = w * 32 + q * 4;
                whole[u] = live && c_of[u] + 3 < cols;
                f[u] = load_input<ONCE>(x + (live ? row : 0) * ld_x + (whole[u] ? c_of[u] : c_last));
                advance(row, w, slice, kw);
            }
#pragma unroll
            for (int u = 0; u < kPackUnroll; ++u) {
                // Out-of-range elements take a negative value: bit 0.
                v[u][0] = whole[u] ? f[u].x : -1.0f;
                v[u][1] = whole[u] ? f[u].y : -1.0f;
                v[u][2] = whole[u] ? f[u].z : -1.0f;
                v[u][3] = whole[u] ? f[u].w : -1.0f;
                if (!whole[u] && row_of[u] >= 0 && c_of[u] < cols) {   // a row's last, partial quad (cols % 4 != 0)
                    const float* p = x + row_of[u] * ld_x + c_of[u];
#pragma unroll
                    for (int e = 0; e < 3; ++e)
                        if (c_of[u] + e < cols) v[u][e] = p[e];
                }
            }
        } else {
#pragma unroll
            for (int u = 0; u < kPackUnroll; ++u) {
                const bool live = g0 + u * kSlice < n_words;
                row_of[u] = live ? row : -1;
                word_of[u] = w;
                const int64_t c0 = w * 32 + q * 4;
                const float* p = x + row * ld_x + c0;
                // Out-of-range elements take a negative value: bit 0.
                v[u][0] = v[u][1] = v[u][2] = v[u][3] = -1.0f;
                if (live) {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c0 + e < cols) v[u][e] = p[e];
                }
                advance(row, w, slice, kw);
            }
        }
#pragma unroll
        for (int u = 0; u < kPackUnroll; ++u) {
            uint32_t nib = ge_zero(v[u][0]) | (ge_zero(v[u][1]) << 1) |
                           (ge_zero(v[u][2]) << 2) | (ge_zero(v[u][3]) << 3);
            const uint32_t word = or_reduce8(nib << (4 * q));
            if (q == 0 && row_of[u] >= 0) out[row_of[u] * ld_out + word_of[u]] = word;
        }
        advance(row0, w0, pass, kw);
    }
}

// Fast path for rows that are whole numbers of 128-element units (see UnitSplit): a group of 8 lanes
// takes 4 consecutive output words, each of its four 16-byte loads per lane covers 128 contiguous bytes
// of the group, and lane 0 writes the four words with one 16-byte store, so a wavefront's store is one
// full 128-byte line instead of four partial ones.
template <bool ONCE>
__global__ __launch_bounds__(kPackThreads) void pack_sign_units_kernel(
    const float* __restrict__ x, int64_t rows, int64_t ld_x, uint32_t* __restrict__ out, int64_t ld_out,
    UnitSplit us) {
    const int q = threadIdx.x & 7, gi = threadIdx.x >> 3;
    const int64_t block_row = int64_t(blockIdx.x) / us.slices_per_row;
    const int slice = int(int64_t(blockIdx.x) - block_row * us.slices_per_row);
    const int unit = us.rows_per_step == 1 ? slice * 32 + gi : gi % us.units_per_row;
    const int row_in_step = us.rows_per_step == 1 ? 0 : gi / us.units_per_row;
    for (int i = 0; i < us.steps; ++i) {
        const int64_t row = (block_row * us.steps + i) * us.rows_per_step + row_in_step;
        if (row >= rows) break;
        const float* p = x + row * ld_x + int64_t(unit) * 128 + q * 4;
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = load_input<ONCE>(p + 32 * u);
        uint32_t w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t nib = ge_zero(v[u].x) | (ge_zero(v[u].y) << 1) | (ge_zero(v[u].z) << 2) | (ge_zero(v[u].w) << 3);
            w[u] = or_reduce8(nib << (4 * q));
        }
        if (q == 0) *reinterpret_cast<uint4*>(out + row * ld_out + int64_t(unit) * 4) = make_uint4(w[0], w[1], w[2], w[3]);
    }
}

// ----------------------------------------------------------------------------
// bnn_pack_bitplanes: 8-bit inputs of the first layer (Sec. 1.6, Alg. 4 step 1) as eight
// packed bit planes.  out[r][8*w + p] holds bit p of x[r][32*w .. 32*w + 31].
//
// Same split as the Sign packer: 8 lanes per 32 elements, 4 bytes per lane.  For plane p the
// lane's four bits sit at bit p of each byte; a multiply gathers them into a nibble
// ((d >> p) & 0x01010101) * 0x10204080 >> 28, the group ORs the shifted nibbles, and lane p
// of the group keeps plane p, so the group's store is 32 contiguous bytes.
// ----------------------------------------------------------------------------
template <bool VEC>
__global__ __launch_bounds__(kPackThreads) void pack_bitplanes_kernel(
    const uint8_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ld_x,
    uint32_t* __restrict__ out, int64_t ld_out, int64_t kw, int64_t n_groups, WordStep st) {
    // One word group per thread group and pass; passes are a whole grid apart (step st).
    const int q = threadIdx.x & 7;
    const int64_t groups_per_pass = int64_t(gridDim.x) * (kPackThreads / 8);
    int64_t g = int64_t(blockIdx.x) * (kPackThreads / 8) + (threadIdx.x >> 3);
    int64_t row = g / kw, w = g - row * kw;
    for (; g < n_groups; g += groups_per_pass) {
        const int64_t c0 = w * 32 + q * 4;
        const uint8_t* p = x + row * ld_x + c0;
        uint32_t d = 0u;                                  // out-of-range elements read as 0: all planes 0
        if (VEC && c0 + 3 < cols) {
            d = *reinterpret_cast<const uint32_t*>(p);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (c0 + e < cols) d |= uint32_t(p[e]) << (8 * e);
        }
        uint32_t mine = 0u;
#pragma unroll
        for (int pl = 0; pl < 8; ++pl) {
            const uint32_t nib = (((d >> pl) & 0x01010101u) * 0x10204080u) >> 28;
            const uint32_t word = or_reduce8(nib << (4 * q));
            if (q == pl) mine = word;
        }
        out[row * ld_out + 8 * w + q] = mine;
        advance(row, w, st, kw);
    }
}

}  // namespace bnn

extern "C" int bnn_pack_bitplanes(const uint8_t* x, int64_t rows, int64_t cols, int64_t ld_x, uint32_t* out,
                                  int64_t ld_out, void* stream) {
    using namespace bnn;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim) return BNN_ERR_INVALID_ARG;
    const int64_t kw = ceil_div(cols, 32);
    if (ld_x < cols || ld_out < 8 * kw) return BNN_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return BNN_OK;
    if (!x || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;
    const int64_t n_groups = rows * kw;
    int64_t blocks = ceil_div(n_groups, kPackThreads / 8);
    if (blocks > 256 * 32) blocks = 256 * 32;
    const bool vec = aligned_to(x, 4) && (ld_x % 4 == 0);
    const WordStep st = word_step(blocks * (kPackThreads / 8), kw);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (vec)
        hipLaunchKernelGGL(pack_bitplanes_kernel<true>, dim3(unsigned(blocks)), dim3(kPackThreads), 0, s, x, rows,
                           cols, ld_x, out, ld_out, kw, n_groups, st);
    else
        hipLaunchKernelGGL(pack_bitplanes_kernel<false>, dim3(unsigned(blocks)), dim3(kPackThreads), 0, s, x, rows,
                           cols, ld_x, out, ld_out, kw, n_groups, st);
    return check_launch();
}

extern "C" int bnn_pack_sign(const float* x, int64_t rows, int64_t cols, int64_t ld_x,
                             uint32_t* out, int64_t ld_out, void* stream) {
    using namespace bnn;
    if (rows < 0 || cols < 0 || rows > kMaxDim || cols > kMaxDim) return BNN_ERR_INVALID_ARG;
    const int64_t kw = ceil_div(cols, 32);
    if (ld_x < cols || ld_out < kw) return BNN_ERR_INVALID_ARG;
    if (rows == 0 || cols == 0) return BNN_OK;
    if (!x || !out) return BNN_ERR_INVALID_ARG;
    if (!aligned_to(x, 4) || !aligned_to(out, 4)) return BNN_ERR_ALIGNMENT;

    const int64_t n_words = rows * kw;
    const int64_t groups_per_block = kPackThreads / 8;
    int64_t blocks = ceil_div(n_words, groups_per_block * kPackUnroll);
    // One pass per workgroup up to 16 GiB of input: measured faster than a smaller grid that loops
    // (1 GiB: 5.98 TB/s in one pass of 65536 workgroups, 5.60 TB/s with 8192 looping 8 times).
    const int64_t max_blocks = int64_t(1) << 20;
    if (blocks > max_blocks) blocks = max_blocks;
    const bool vec = aligned_to(x, 16) && (ld_x % 4 == 0);
    const bool once = rows * cols * int64_t(sizeof(float)) > kOnceMinBytes;     // see load_input
    hipStream_t s = static_cast<hipStream_t>(stream);
    UnitSplit us;
    if (vec && aligned_to(out, 16) && ld_out % 4 == 0 && unit_split(cols, 1, us)) {
        const int64_t unit_blocks = ceil_div(rows, int64_t(us.rows_per_step) * us.steps) * us.slices_per_row;
        if (unit_blocks <= kMaxDim) {
            if (once)
                hipLaunchKernelGGL(pack_sign_units_kernel<true>, dim3(unsigned(unit_blocks)), dim3(kPackThreads), 0, s, x, rows,
                                   ld_x, out, ld_out, us);
            else
                hipLaunchKernelGGL(pack_sign_units_kernel<false>, dim3(unsigned(unit_blocks)), dim3(kPackThreads), 0, s, x, rows,
                                   ld_x, out, ld_out, us);
            return check_launch();
        }
    }
    const WordStep slice = word_step(groups_per_block, kw);
    const WordStep pass = word_step(blocks * groups_per_block * kPackUnroll, kw);
    if (vec && once)
        hipLaunchKernelGGL((pack_sign_kernel<true, true>), dim3(unsigned(blocks)), dim3(kPackThreads), 0, s,
                           x, rows, cols, ld_x, out, ld_out, kw, n_words, slice, pass);
    else if (vec)
        hipLaunchKernelGGL((pack_sign_kernel<true, false>), dim3(unsigned(blocks)), dim3(kPackThreads), 0, s,
                           x, rows, cols, ld_x, out, ld_out, kw, n_words, slice, pass);
    else
        hipLaunchKernelGGL((pack_sign_kernel<false, false>), dim3(unsigned(blocks)), dim3(kPackThreads), 0, s,
                           x, rows, cols, ld_x, out, ld_out, kw, n_words, slice, pass);
    return check_launch();
}
