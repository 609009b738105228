// Binary "same" convolution (stride 1, output size = input size, kh = kw = 2*pad + 1: the 3 x 3,
// pad 1 layers of the paper's ConvNets, Sec. 3.3) with the input patch of a tile resident in LDS.
//
// The GEMM view of the layer is C[pixel][filter] = XnorDotProduct(receptive field, filter) (Alg. 4)
// with K = kh*kw*Cin.  The receptive fields of neighbouring pixels overlap kh*kw-fold, so instead
// of staging every K-tile of the (implicit) im2col matrix, a workgroup loads each input pixel its
// tile needs ONCE: a tile is BM consecutive output pixels = R whole image rows (or R / H whole
// images), its patch those rows plus a halo of `pad` pixels all around, kept in LDS for the
// workgroup's life.  Halo cells outside the image hold all-ones words (+1, zero padding through
// Eq. (1)).  The A operand of an MFMA step for tap (ky, kx) is then a plain LDS read at
//     slot(pixel) + ky * PW + kx          (PW = W + 2*pad, patch row pitch in pixels)
// with no per-tap bounds logic, and only the filters (B) stream through LDS K-tile by K-tile.
// Arithmetic, widening, fix-up and epilogues are those of xnor_gemm_mfma.hip; the row popcounts are
// sums of per-pixel popcounts over the taps.
//
// Patch layout: planes [channel quad cq][half h] of 8-byte slots, slot s = words 4*cq + 2*h, +1 of
// patch pixel s; lanes of an operand read consecutive pixels, hence consecutive slots.
// B K-tile layout: planes [quad][half] of 8-byte slots, as in the short-K kernel.
//
// Pooled layers (POOL = true): the paper's ConvNets max-pool the pre-activations 2 x 2 between a
// convolution and its BatchNorm + Sign.  Sign(BatchNorm(.)) is monotone per channel, so the pooled
// output bit is the OR of the window's four output bits where the folded flip bit is 0 and their
// AND where it is 1.  A tile holds whole (even numbers of) image rows, so every window lies inside
// one wavefront's rows: the horizontal neighbour is the next lane, the vertical one W lanes away
// (W < 32) or in the accumulator block W / 32 further on, and only the pooled words are stored.
//
// Channel counts that are multiples of 32 but not of 128 (WORDS = true; the 64-channel block of the
// half-width SVHN net of Sec. 2.3): a tap is then not a whole number of 16-byte quads, so the patch is
// kept as planes [channel word][slot] of single words, and the K-word that lane half h consumes at step
// (quad q, s), word 4q + 2h + s of the receptive field, is looked up in a small LDS table that maps
// a K-word to (channel word plane, tap offset).  Filter words beyond the receptive field's last word
// are zeroed at staging.  Everything else is shared.
//
// Geometry this kernel takes (the launcher checks; everything else goes to the gathering kernels):
// stride 1, Ho = H, Wo = W, Cin % 32 == 0, BM % W == 0 and, with R = BM / W, H % R == 0 or
// R % H == 0; filters 16-byte aligned with ldb % 4 == 0; patch within kPatchMaxBytes of LDS; with
// Cin % 128 != 0 a receptive field of at most kResidentKTiles * 512 bits.
#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {

constexpr int kPatchMaxBytes = 40 * 1024;

struct PatchGeom {
    int groups;        // images (or row blocks) in a tile
    int rows;          // output rows per group
    int prows, pw;     // patch rows per group, patch row pitch (pixels)
    int slots;         // groups * prows * pw
    int cqn;           // channel quads per pixel (Cw / 4); unused when a tap is not a whole number of quads
    int kq;            // quads of K per filter row: kh * kw * cqn, or ceil(kwords / 4)
    int kwords;        // words of K per filter row: kh * kw * Cw
};

// Word offset of the K-word table behind the word-granular patch ([Cw][slots] words + slots pixel popcounts).
__host__ __device__ inline size_t words_patch_koff_offset(int Cw, int slots) {
    return (size_t(Cw + 1) * size_t(slots) + 1) & ~size_t(1);
}

// BRES: the filters' whole K extent (at most kResidentKTiles K-tiles of 4 quads) is staged once, next
// to the patch, and the K loop runs without a barrier; otherwise B streams through two K-tile buffers.
constexpr int kResidentKTiles = 5;

template <int WM, bool FUSED, bool POOL, bool BRES, bool WORDS>
__global__ __launch_bounds__(256, WM >= 4 ? 2 : 3) void conv_patch_mfma_kernel(
    const uint32_t* __restrict__ in, const uint32_t* __restrict__ B, int64_t ldb, int32_t* __restrict__ C,
    int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn, ConvArgs cv, PatchGeom pg,
    int n_images) {
    constexpr int WN = 2, BM = 64 * WM, BN = 64 * WN;
    constexpr int PLANE_B = BN + 2;                     // 8-byte slots per B plane (2 pad slots)
    constexpr int ST_ROWS = 256 / 4;                    // filter rows per staging pass (4 threads per row)
    constexpr int LOADS_B = BN / ST_ROWS;
    static_assert(!WORDS || BRES, "the word-granular patch is built for resident filters only");
    extern __shared__ uint2 patch[];                    // [cqn][2][slots], int pix_pop[slots], resident B tiles
                                                        // WORDS: uint32 [Cw][slots], pix_pop, int koff[4*kq], B tiles
    __shared__ uint2 lds_b_stream[BRES ? 1 : 2 * 8 * PLANE_B];
    __shared__ __attribute__((aligned(16))) int pop_a[BM];
    __shared__ __attribute__((aligned(16))) float pop_af[FUSED ? BM : 4];
    __shared__ __attribute__((aligned(16))) int pop_b[BN];
    __shared__ __attribute__((aligned(16))) int thr_s[FUSED ? BN : 1];
    __shared__ uint32_t flip_s[FUSED ? BN / 32 : 1];
    __shared__ float colfix_s[FUSED ? BN : 1];
    __shared__ int coord_s[BM];
    uint32_t* patchw = reinterpret_cast<uint32_t*>(patch);
    int* pix_pop = WORDS ? reinterpret_cast<int*>(patchw + size_t(cv.Cw) * pg.slots)
                         : reinterpret_cast<int*>(patch + size_t(2) * pg.cqn * pg.slots);
    // WORDS: K-word -> plane and tap offset into patchw, read two at a time (hence the even word offset)
    const size_t koff_at = words_patch_koff_offset(cv.Cw, pg.slots);
    int* koff_s = reinterpret_cast<int*>(patchw) + koff_at;
    uint2* lds_b = !BRES ? lds_b_stream                 // [buffer][8 planes]
                   : WORDS ? patch + (koff_at + size_t(4) * pg.kq) / 2
                           : patch + size_t(2) * pg.cqn * pg.slots + (pg.slots + 1) / 2;

    int tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int row0 = tile_m * BM, col0 = tile_n * BN;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;

    // ---- B staging: K-tiles of 4 quads, as planes [quad][half] ---------------------------------
    const int st_q = tid & 3, st_r = tid >> 2;
    const uint32_t* pb[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) pb[l] = B + int64_t(min(col0 + st_r + l * ST_ROWS, N - 1)) * ldb;
    uint4 rb[LOADS_B];
    int cnt_b[LOADS_B];
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) cnt_b[l] = 0;
    const int n_ktiles = (pg.kq + 3) >> 2;
    auto fetch_b = [&](int kt) {
        const int quad = min(4 * kt + st_q, pg.kq - 1);           // clamped; zeroed at staging if past the row
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) rb[l] = *reinterpret_cast<const uint4*>(pb[l] + 4 * quad);
    };
    auto stage_b = [&](int kt, int buf) {
        const bool live = 4 * kt + st_q < pg.kq;
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            uint4 v = zero_unless(live, rb[l]);
            if (WORDS) {                                // words of the quad beyond the receptive field's last one
                const int left = pg.kwords - 4 * (4 * kt + st_q);
                if (left < 4) v.w = 0u;
                if (left < 3) v.z = 0u;
                if (left < 2) v.y = 0u;
            }
            cnt_b[l] += popc4(v);
            lds_b[(8 * buf + 2 * st_q) * PLANE_B + st_r + l * ST_ROWS] = make_uint2(v.x, v.y);
            lds_b[(8 * buf + 2 * st_q + 1) * PLANE_B + st_r + l * ST_ROWS] = make_uint2(v.z, v.w);
        }
    };

    // Output pixel r of the tile as (group, row in group, column), 10 bits each: the divisions are done
    // once per pixel here, not once per use.
    if (tid < BM) {
        const int per_group = pg.rows * cv.W;
        const int g = tid / per_group, t = tid - g * per_group;
        const int yl = t / cv.W, x = t - yl * cv.W;
        coord_s[tid] = (g << 20) | (yl << 10) | x;
    }
    // Thresholds and flip words go to registers here and to LDS after the patch loads have been issued: every
    // global load of the prologue (these, the filters, the patch) is in flight before the first one is waited for.
    int thr_reg = 0;
    uint32_t flip_reg = 0u;
    if (FUSED) {
        if (tid < BN && col0 + tid < N) thr_reg = bn.thr[col0 + tid];
        if (tid < BN / 32 && col0 + 32 * tid < N) flip_reg = bn.flip_bits[(col0 >> 5) + tid];
    }
    // The filter loads are issued first, so that they are in flight while the patch is addressed and loaded.
    uint4 all_b[BRES ? kResidentKTiles : 1][LOADS_B];
    if (BRES) {
#pragma unroll
        for (int kt = 0; kt < kResidentKTiles; ++kt)
            if (kt < n_ktiles) {
                fetch_b(kt);
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l) all_b[kt][l] = rb[l];
            }
    } else {
        fetch_b(0);
    }

    // ---- patch: every slot once ------------------------------------------------------------
    // The tile's first output pixel is (image b0, row y0, column 0); group g covers image rows
    // y0 .. y0 + rows - 1 of image b0 (one group) or all rows of image b0 + g (several groups).
    const int hw = cv.H * cv.W;
    const int b0 = row0 / hw, y0 = (row0 - b0 * hw) / cv.W;
    const int group_slots = pg.prows * pg.pw;
    if (WORDS || !FUSED) {
        // Slot by slot (the word-granular patch, and the int32 form, whose epilogue leaves no registers for
        // more loads in flight).
        for (int s = tid; s < pg.slots; s += 256) {
            const int g = s / group_slots, t = s - g * group_slots;
            const int py = t / pg.pw, px = t - py * pg.pw;
            const int b = b0 + g, y = y0 + py - cv.pad, x = px - cv.pad;
            const bool inside = b < n_images && y >= 0 && y < cv.H && x >= 0 && x < cv.W;
            const uint32_t pix = inside ? uint32_t((b * cv.H + y) * cv.W + x) : 0u;
            const uint32_t* p = in + size_t(pix) * uint32_t(cv.Cw);
            int pop = 0;
            if (WORDS) {
                for (int cw = 0; cw < cv.Cw; ++cw) {
                    const uint32_t v = inside ? p[cw] : ~0u;
                    patchw[cw * pg.slots + s] = v;
                    pop += __popc(v);
                }
            } else {
                for (int cq = 0; cq < pg.cqn; ++cq) {
                    uint4 v = *reinterpret_cast<const uint4*>(p + 4 * cq);
                    if (!inside) v = make_uint4(~0u, ~0u, ~0u, ~0u);
                    patch[(2 * cq) * pg.slots + s] = make_uint2(v.x, v.y);
                    patch[(2 * cq + 1) * pg.slots + s] = make_uint2(v.z, v.w);
                    pop += popc4(v);
                }
            }
            pix_pop[s] = pop;
        }
    } else {
        // Two slots per thread and pass, up to four channel quads of each at a time: all (up to eight) loads
        // of a pass are issued before the first LDS write waits for one.  Slots that do not exist and cells
        // outside the image load input pixel 0 (a valid address) and are not written / written as all ones.
        constexpr int kSlotsPerPass = 2, kQuadsPerPass = 4;
        for (int s_base = 0; s_base < pg.slots; s_base += kSlotsPerPass * 256) {
            const uint32_t* p[kSlotsPerPass];
            bool live[kSlotsPerPass], inside[kSlotsPerPass];
            int pop[kSlotsPerPass];
#pragma unroll
            for (int u = 0; u < kSlotsPerPass; ++u) {
                const int s = s_base + u * 256 + tid;
                live[u] = s < pg.slots;
                const int g = s / group_slots, t = s - g * group_slots;
                const int py = t / pg.pw, px = t - py * pg.pw;
                const int b = b0 + g, y = y0 + py - cv.pad, x = px - cv.pad;
                inside[u] = live[u] && b < n_images && y >= 0 && y < cv.H && x >= 0 && x < cv.W;
                const uint32_t pix = inside[u] ? uint32_t((b * cv.H + y) * cv.W + x) : 0u;
                p[u] = in + size_t(pix) * uint32_t(cv.Cw);
                pop[u] = 0;
            }
            for (int cq0 = 0; cq0 < pg.cqn; cq0 += kQuadsPerPass) {
                uint4 v[kSlotsPerPass][kQuadsPerPass];
#pragma unroll
                for (int u = 0; u < kSlotsPerPass; ++u)
#pragma unroll
                    for (int c = 0; c < kQuadsPerPass; ++c)
                        if (cq0 + c < pg.cqn) v[u][c] = *reinterpret_cast<const uint4*>(p[u] + 4 * (cq0 + c));
#pragma unroll
                for (int u = 0; u < kSlotsPerPass; ++u) {
                    const int s = s_base + u * 256 + tid;
#pragma unroll
                    for (int c = 0; c < kQuadsPerPass; ++c)
                        if (cq0 + c < pg.cqn) {
                            const uint4 w = inside[u] ? v[u][c] : make_uint4(~0u, ~0u, ~0u, ~0u);
                            if (live[u]) {
                                patch[(2 * (cq0 + c)) * pg.slots + s] = make_uint2(w.x, w.y);
                                patch[(2 * (cq0 + c) + 1) * pg.slots + s] = make_uint2(w.z, w.w);
                            }
                            pop[u] += popc4(w);
                        }
                }
            }
#pragma unroll
            for (int u = 0; u < kSlotsPerPass; ++u)
                if (live[u]) pix_pop[s_base + u * 256 + tid] = pop[u];
        }
    }
    if (FUSED) {
        if (tid < BN) thr_s[tid] = max(-K - 1, min(K + 1, thr_reg));
        if (tid < BN / 32) flip_s[tid] = flip_reg;
    }
    if (WORDS) {
        // K-word kwi of a receptive field = channel word kwi % Cw of tap kwi / Cw; words past the field's
        // end point at a valid cell (their filter words are zero).
        for (int kwi = tid; kwi < 4 * pg.kq; kwi += 256) {
            int off = 0;
            if (kwi < pg.kwords) {
                const int tap = kwi / cv.Cw, cw = kwi - tap * cv.Cw;
                const int ty = tap / cv.kw, tx = tap - ty * cv.kw;
                off = cw * pg.slots + ty * pg.pw + tx;
            }
            koff_s[kwi] = off;
        }
    }

    if (BRES) {
#pragma unroll
        for (int kt = 0; kt < kResidentKTiles; ++kt)
            if (kt < n_ktiles) {
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l) rb[l] = all_b[kt][l];
                stage_b(kt, kt);
            }
    } else {
        stage_b(0, 0);
    }
    __syncthreads();                                    // patch, pixel popcounts and the first (or every) B tile are in LDS

    // Row popcounts: sum of the pixel popcounts under the kh x kw window (read before the epilogue,
    // which follows at least one more barrier).
    auto slot_of = [&](int r) {
        const int c = coord_s[r];
        return (c >> 20) * group_slots + ((c >> 10) & 1023) * pg.pw + (c & 1023);
    };
    if (tid < BM) {
        const int s0 = slot_of(tid);
        int sum = 0;
        for (int ky = 0; ky < cv.kh; ++ky)
            for (int kx = 0; kx < cv.kw; ++kx) sum += pix_pop[s0 + ky * pg.pw + kx];
        pop_a[tid] = 2 * sum;
        if (FUSED) pop_af[tid] = 0.5f * float(sum);
    }

    // This lane's A operands: pixel wm*32*WM + i*32 + fr, words of lane half fh.
    const uint2* rd_a[WM];
    const uint32_t* rd_aw[WM];                          // WORDS: the pixel's cell in plane 0
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int slot = slot_of(wm * 32 * WM + i * 32 + fr);
        rd_a[i] = patch + fh * pg.slots + slot;
        rd_aw[i] = patchw + slot;
    }
    const int rd_b = fh * PLANE_B + wn * 32 * WN + fr;

    v16f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // (tap row, tap column, channel quad) of the next quad of K, stepped with carries.
    int ky = 0, kx = 0, cq = 0;
    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int buf = BRES ? kt : kt & 1;
        if (!BRES && kt + 1 < n_ktiles) fetch_b(kt + 1);
        const int quads_here = min(4, pg.kq - 4 * kt);
#pragma unroll
        for (int qq = 0; qq < 4; ++qq) {
            if (qq >= quads_here) break;
            uint2 aw[WM], bw[WN];
            if (WORDS) {
                // this lane half's two K-words of the quad: 4q + 2*fh and the next one
                const int2 off = *reinterpret_cast<const int2*>(&koff_s[4 * (4 * kt + qq) + 2 * fh]);
#pragma unroll
                for (int i = 0; i < WM; ++i) aw[i] = make_uint2(rd_aw[i][off.x], rd_aw[i][off.y]);
            } else {
                const int a_off = (2 * cq) * pg.slots + ky * pg.pw + kx;
#pragma unroll
                for (int i = 0; i < WM; ++i) aw[i] = rd_a[i][a_off];
            }
#pragma unroll
            for (int j = 0; j < WN; ++j) bw[j] = lds_b[(8 * buf + 2 * qq) * PLANE_B + rd_b + j * 32];
#pragma unroll
            for (int s = 0; s < 2; ++s) {
                v8i fa[WM], fb[WN];
#pragma unroll
                for (int i = 0; i < WM; ++i) fa[i] = widen_fp4_a(s == 0 ? aw[i].x : aw[i].y);
#pragma unroll
                for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(s == 0 ? bw[j].x : bw[j].y);
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) {
                        // fused: operands swapped, the accumulators hold the transposed blocks (mfma_epilogue_bits)
                        if (FUSED)
                            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                fb[j], fa[i], acc[i][j], 4 /* fp4 */, 4 /* fp4 */, 0, 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                fa[i], fb[j], acc[i][j], 4 /* A: fp4 */, 4 /* B: fp4 */, 0, 0, 0, 0);
                    }
            }
            if (!WORDS && ++cq == pg.cqn) {
                cq = 0;
                if (++kx == cv.kw) {
                    kx = 0;
                    ++ky;
                }
            }
        }
        if (!BRES) {
            // Keep the staging of the next B tile (and the wait for its loads) behind the MFMA steps.
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j) asm volatile("" : "+v"(acc[i][j]) : : "memory");
            if (kt + 1 < n_ktiles) stage_b(kt + 1, buf ^ 1);
            __syncthreads();
        }
    }

#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) {
        int c = cnt_b[l];
        c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);       // lane ^ 1
        c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);       // lane ^ 2
        if (st_q == 0) {
            pop_b[st_r + l * ST_ROWS] = 2 * c;
            if (FUSED) colfix_s[st_r + l * ST_ROWS] = fold_column_term(thr_s[st_r + l * ST_ROWS], K, 2 * c);
        }
    }
    __syncthreads();

    if constexpr (POOL) {
        static_assert(FUSED, "pooling acts on output bits");
        uint32_t words[WM];
        mfma_output_words<WM, WN>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, colfix_s, N, K, col0, wm, wn, fr, fh, words);
        const uint32_t flip_word = flip_s[wn * WN + fh];
        const int64_t nw = (int64_t(N) + 31) >> 5;
        const int64_t w = ((int64_t(col0) + wn * 32 * WN) >> 5) + fh;
        uint32_t any[WM], all[WM];
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            // horizontal neighbour (x ^ 1): the next lane; vertical one for W < 32: W lanes away
            const uint32_t h = uint32_t(__shfl_xor(int(words[i]), 1));
            any[i] = words[i] | h;
            all[i] = words[i] & h;
            if (cv.W < 32) {
                any[i] |= uint32_t(__shfl_xor(int(any[i]), cv.W));
                all[i] &= uint32_t(__shfl_xor(int(all[i]), cv.W));
            }
        }
        const int blocks_per_row = cv.W >> 5;           // W >= 32: image row y and y + 1 are blocks i and i + W / 32
        const int hp = cv.H >> 1, wp = cv.W >> 1;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            uint32_t a = any[i], l = all[i];
            if (cv.W >= 32) {
#pragma unroll
                for (int i2 = 0; i2 < WM; ++i2)
                    if (i2 == i + blocks_per_row) {
                        a |= any[i2];
                        l &= all[i2];
                    }
            }
            const int rl = wm * 32 * WM + i * 32 + fr, m = row0 + rl;
            const int c = coord_s[rl];
            const int b = b0 + (c >> 20), y = y0 + ((c >> 10) & 1023), x = c & 1023;
            const uint32_t pooled = (a & ~flip_word) | (l & flip_word);
            if (m < M && w < nw && !(y & 1) && !(x & 1))
                bn.out[(int64_t(b) * hp + (y >> 1)) * wp * bn.ld_out + int64_t(x >> 1) * bn.ld_out + w] = pooled;
        }
    } else if constexpr (FUSED)
        mfma_epilogue_bits<WM, WN>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, colfix_s, bn, M, N, K, row0, col0, wm, wn,
                                   fr, fh);
    else
        mfma_epilogue<WM, WN, false, false>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, C, ldc, bn, M, N, K, row0, col0,
                                            wm, wn, fr, fh);
}

// Fills the patch geometry for tiles of BM output pixels; false if this convolution does not fit.
static bool patch_geometry(const ConvArgs& cv, int BM, PatchGeom& pg) {
    if (cv.stride != 1 || cv.Ho != cv.H || cv.Wo != cv.W) return false;
    if (cv.kh != 2 * cv.pad + 1 || cv.kw != 2 * cv.pad + 1) return false;
    if (cv.W > BM || BM % cv.W != 0) return false;
    const int R = BM / cv.W;
    if (cv.H % R == 0) {
        pg.groups = 1;
        pg.rows = R;
    } else if (R % cv.H == 0) {
        pg.groups = R / cv.H;
        pg.rows = cv.H;
    } else {
        return false;
    }
    pg.prows = pg.rows + 2 * cv.pad;
    pg.pw = cv.W + 2 * cv.pad;
    pg.slots = pg.groups * pg.prows * pg.pw;
    pg.cqn = cv.Cw / 4;
    pg.kwords = cv.kh * cv.kw * cv.Cw;
    pg.kq = (pg.kwords + 3) / 4;
    if (cv.Cw % 4 != 0 && (pg.kq + 3) / 4 > kResidentKTiles) return false;     // word-granular patch: resident filters only
    return int64_t(pg.slots) * (cv.Cw * 4 + 4) <= kPatchMaxBytes;
}

template <int WM, bool FUSED, bool POOL>
static int launch_patch(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                        int64_t N, int64_t K, BnSignArgs bn, ConvArgs cv, PatchGeom pg, void* stream) {
    const int64_t tiles_m = ceil_div(M, 64 * WM), tiles_n = ceil_div(N, 128);
    if (tiles_m * tiles_n > kMaxDim) return BNN_ERR_UNSUPPORTED;
    const bool words = cv.Cw % 4 != 0;                  // a tap is not a whole number of 16-byte quads
    const size_t patch_bytes = words ? (words_patch_koff_offset(cv.Cw, pg.slots) + size_t(4) * pg.kq) * 4
                                     : size_t(pg.slots) * size_t(cv.Cw) * 4 + size_t((pg.slots + 1) / 2) * 8;
    const int n_ktiles = (pg.kq + 3) / 4;
    const bool resident = n_ktiles <= kResidentKTiles;
    const size_t lds_bytes = patch_bytes + (resident ? size_t(n_ktiles) * 8 * (128 + 2) * sizeof(uint2) : 0);
    const int n_images = int(M / (int64_t(cv.H) * cv.W));
    const dim3 grid(unsigned(tiles_m * tiles_n));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (words)                                          // patch_geometry has checked that the filters are resident
        hipLaunchKernelGGL((conv_patch_mfma_kernel<WM, FUSED, POOL, true, true>), grid, dim3(256), lds_bytes, s, in, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn, cv, pg, n_images);
    else if (resident)
        hipLaunchKernelGGL((conv_patch_mfma_kernel<WM, FUSED, POOL, true, false>), grid, dim3(256), lds_bytes, s, in, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn, cv, pg, n_images);
    else
        hipLaunchKernelGGL((conv_patch_mfma_kernel<WM, FUSED, POOL, false, false>), grid, dim3(256), lds_bytes, s, in, B,
                           ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn, cv, pg, n_images);
    return check_launch();
}

// BNN_ERR_UNSUPPORTED if the geometry is not one this kernel takes (the caller then uses the
// gathering kernels).  Tile choice as for the plain product: 256 pixels x 128 filters when that grid
// fills the chip's 512 workgroup slots, else 128 x 128.
template <bool FUSED>
static int launch_conv_patch_any(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc,
                                 int64_t M, int64_t N, int64_t K, BnSignArgs bn, ConvArgs cv, void* stream) {
    if (!aligned_to(B, 16) || ldb % 4 != 0) return BNN_ERR_UNSUPPORTED;
    PatchGeom pg;
    const bool big = ceil_div(M, 256) * ceil_div(N, 128) >= 512;
    if (big && patch_geometry(cv, 256, pg))
        return launch_patch<4, FUSED, false>(in, B, ldb, C, ldc, M, N, K, bn, cv, pg, stream);
    if (patch_geometry(cv, 128, pg)) return launch_patch<2, FUSED, false>(in, B, ldb, C, ldc, M, N, K, bn, cv, pg, stream);
    return BNN_ERR_UNSUPPORTED;
}

// 2 x 2 pooling inside a tile of BM = 64 * WM pixels: even H and W, W a power of two below 32 or 32 * k
// with the row pair inside one wavefront's WM blocks, and an even number of image rows per tile.
static bool pool_fits(const ConvArgs& cv, const PatchGeom& pg, int WM) {
    if ((cv.H & 1) || (cv.W & 1) || (pg.rows & 1)) return false;
    if (cv.W < 32) return (cv.W & (cv.W - 1)) == 0;
    return cv.W % 32 == 0 && 2 * (cv.W / 32) <= WM;
}

int launch_conv_patch(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                      int64_t N, int64_t K, ConvArgs cv, void* stream) {
    return launch_conv_patch_any<false>(in, B, ldb, C, ldc, M, N, K, BnSignArgs{}, cv, stream);
}

int launch_conv_patch_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                            BnSignArgs bn, ConvArgs cv, void* stream) {
    return launch_conv_patch_any<true>(in, B, ldb, nullptr, 0, M, N, K, bn, cv, stream);
}

// Convolution, 2 x 2 max pooling (stride 2), BatchNorm, Sign in one launch; bn.out is the pooled
// packed NHWC map [B][H/2][W/2][ld_out].  BNN_ERR_UNSUPPORTED where the pooling windows do not fit
// the tiles (the caller then pools the unpooled output bits with bnn_maxpool_bits).
int launch_conv_patch_pool_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                                 BnSignArgs bn, ConvArgs cv, void* stream) {
    if (!aligned_to(B, 16) || ldb % 4 != 0) return BNN_ERR_UNSUPPORTED;
    PatchGeom pg;
    const bool big = ceil_div(M, 256) * ceil_div(N, 128) >= 512;
    if (big && patch_geometry(cv, 256, pg) && pool_fits(cv, pg, 4))
        return launch_patch<4, true, true>(in, B, ldb, nullptr, 0, M, N, K, bn, cv, pg, stream);
    if (patch_geometry(cv, 128, pg) && pool_fits(cv, pg, 2))
        return launch_patch<2, true, true>(in, B, ldb, nullptr, 0, M, N, K, bn, cv, pg, stream);
    if (patch_geometry(cv, 256, pg) && pool_fits(cv, pg, 4))
        return launch_patch<4, true, true>(in, B, ldb, nullptr, 0, M, N, K, bn, cv, pg, stream);
    return BNN_ERR_UNSUPPORTED;
}

}  // namespace bnn
