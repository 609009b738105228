// Bits-in, matrix-engine-inside kernels for the products of Alg. 4:
//
//   binary  (PLANES = false)  a_k = XnorDotProduct(a^b_{k-1}, W^b_k), Sec. 4 Eq. (5)
//   planes  (PLANES = true)   a_1 = sum_{n=1..8} 2^(n-1) * <a_0^n, W^b_1>, Alg. 4 step 1 /
//                             Sec. 1.6: 8-bit inputs as eight bit planes a_0^n in {0,1}
//   conv    (CONV = true)     the binary product whose A rows are the receptive fields of a
//                             kh x kw convolution (3 x 3 in the paper's nets, Sec. 3.3), gathered
//                             from the packed NHWC input while the tile is staged (implicit
//                             GEMM: the im2col matrix is never written); taps outside the image
//                             are +1, i.e. all-ones words (zero padding through Eq. (1))
//
// Operands stay packed 32 per word in HBM and LDS (the 32x smaller footprint the
// paper argues for); only inside registers is each bit widened to a 4-bit float
// and fed to v_mfma_f32_32x32x64_f8f6f4 (its block-scaled form in the planes
// kernel), whose fp32 accumulation of small integers is exact below 2^24.  With a, b in {0,1} standing for -1/+1:
//
//   binary:  sum_k (2a-1)(2b-1) = K - 2*popcount(A_m) - 2*popcount(B_n) + 4 * sum_k a*b
//   planes:  sum_n 2^(n-1) sum_k x^n (2b-1) = 2 * sum_n 2^(n-1) sum_k x^n b  -  sum_k x[m][k]
//
// so each product is the matrix-engine sum S plus row (and column) popcounts, which
// the staging threads gather for free while they copy the tile.  In the planes
// kernel the weight 2^(n-1) is the MFMA's block scale of the A operand (E8M0
// exponent 127 + n - 1), so all eight planes accumulate into the same registers.
// Pad bits and words beyond K are zeroed at staging and therefore contribute to
// neither S nor the popcounts; tile rows beyond the matrix are computed on a copy
// of its last row and never stored.
//
// Widening: element k of a word lands in operand register k%4, nibble k/4, for
// both operands (the sum over k does not depend on its order).  The E2M1 codes
// 0b0001, 0b0010, 0b0100 are 0.5, 1.0, 2.0, so most registers are a bare mask of
// the word and only the product of the two sides has to be 1:
//   register   0                      1                  2                        3
//   A side     w & 0x1111.. (0.5)     w & 0x2222.. (1)   w & 0x4444.. (2)         (w>>2) & 0x2222.. (1)
//   B side     (w<<2) & 0x4444.. (2)  w & 0x2222.. (1)   (w>>2) & 0x1111.. (0.5)  (w>>2) & 0x2222.. (1)
// i.e. 5 vector-ALU operations per 32 elements on the A side, 6 on the B side.
//
// Workgroup = 256 threads = 2 x 2 wavefronts; a wavefront owns WM x WN blocks
// of 32 x 32 outputs (fp32 accumulators).  A advances 16 words per staged tile =
// 8 MFMA steps: lane (row r = l%32, half h = l/32) of a fragment owns words
// [8h, 8h+8) of its tile row, read with two ds_read_b128.
//   binary: those 16 words are 512 consecutive bits of K; B is staged the same way.
//   planes: A rows are [K/32 words][8 planes] (word index 8*w + p), so a tile is two
//           K-words x 8 planes, lane half h owns K-word 2*kt + h, step s is plane s;
//           B contributes one word per lane half and tile, widened once per tile.
// The tile is long enough that the global loads of the next tile, issued
// before the MFMA steps, have landed when they are staged.
#include "bnn_internal.h"
#include "gemm_staging.h"
#include "mfma_fp4.h"

namespace bnn {

template <int WM, int WN, bool VEC, bool FUSED, bool PLANES, bool CONV>
__global__ __launch_bounds__(256, WM >= 4 ? 2 : 3) void xnor_gemm_mfma_kernel(
    const uint32_t* __restrict__ A, int64_t lda, const uint32_t* __restrict__ B, int64_t ldb,
    int32_t* __restrict__ C, int64_t ldc, int M, int N, int K, int tiles_m, int tiles_n, BnSignArgs bn,
    ConvArgs cv) {
    static_assert(!(PLANES && CONV), "one A layout at a time");
    constexpr int BM = 64 * WM, BN = 64 * WN;          // 2 x 2 wavefronts
    constexpr int PLANE_A = BM + 2, PLANE_B = BN + 2;  // 16-byte slots per quad plane (2 pad slots)
    constexpr int ST_ROWS = 256 / kMfmaKQ;             // rows covered by one staging pass
    constexpr int LOADS_A = BM / ST_ROWS;
    constexpr int LOADS_B = PLANES ? 0 : BN / ST_ROWS;
    constexpr int NB = PLANES ? 1 : LOADS_B;           // array extent (arrays of length 0 are not allowed)
    static_assert(BM % ST_ROWS == 0 && BN % ST_ROWS == 0, "tile rows must divide among the staging threads");
    static_assert(kMfmaKQ == 4, "the row-popcount reduction below assumes 4 staging lanes per row");
    static_assert(!PLANES || BN * 2 == 256, "the planes kernel stages one B word per thread");
    __shared__ uint4 lds_a[2][kMfmaKQ * PLANE_A];
    __shared__ uint4 lds_b[PLANES ? 1 : 2][PLANES ? 1 : kMfmaKQ * PLANE_B];
    __shared__ uint32_t lds_bw[PLANES ? 2 : 1][PLANES ? 2 * BN : 1];     // planes: [buf][half][row]
    __shared__ __attribute__((aligned(16))) int pop_a[BM];
    __shared__ __attribute__((aligned(16))) int pop_b[BN];
    __shared__ __attribute__((aligned(16))) float pop_af[FUSED ? BM : 4];   // row term of the float threshold
    __shared__ __attribute__((aligned(16))) int thr_s[FUSED ? BN : 1];                  // the tile's thresholds and flip words, fetched
    __shared__ uint32_t flip_s[FUSED ? BN / 32 : 1];       // before the K loop (read in the epilogue)
    // The fused binary kernel multiplies with the operands swapped: its accumulator blocks are the
    // transposes of the output blocks, which lets the epilogue pack a row's bits inside a lane.
    constexpr bool BITS = FUSED && !PLANES;
    __shared__ float colfix_s[BITS ? BN : 1];              // column term of the folded threshold

    int tile_m, tile_n;
    tile_of_block(blockIdx.x, tiles_m, tiles_n, tile_m, tile_n);
    const int row0 = tile_m * BM, col0 = tile_n * BN;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int fr = lane & 31, fh = lane >> 5;
    const int kw = (K + 31) >> 5;                      // words of K per B row (and per plane of A)
    const int kwa = PLANES ? 8 * kw : kw;              // words per A row
    const uint32_t tmask = tail_mask(K);
    const int n_ktiles = (kwa + kMfmaKT - 1) / kMfmaKT;
    // K-tiles made only of complete, unmasked words take branch-free loads (row index clamped
    // into the matrix, result zeroed at staging if the row does not exist); the last, partial
    // K-tile goes through checked, masking loads.
    const int n_full_ktiles = PLANES ? (K >> 5) / 2 : (K >> 5) / kMfmaKT;

    const int st_q = tid % kMfmaKQ, st_r = tid / kMfmaKQ;
    // conv: per staged row the word offset of its image and its output pixel (oy << 16 | ox);
    // otherwise the row pointer.  fill_a: what staging writes for a fetched quad
    // (0 = the loaded words, 1 = all ones: tap outside the image, 2 = zeros: no such row or word).
    const uint32_t* pa[LOADS_A];
    uint32_t img_off[LOADS_A];
    int pix[LOADS_A];
    bool live_a[LOADS_A];
    int fill_a[LOADS_A];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) {
        const int r = row0 + st_r + l * ST_ROWS;
        live_a[l] = r < M;
        fill_a[l] = 0;
        const int rc = min(r, M - 1);
        if (CONV) {
            const int ox = rc % cv.Wo, t = rc / cv.Wo;
            const int oy = t % cv.Ho, b = t / cv.Ho;
            img_off[l] = uint32_t(b) * uint32_t(cv.H * cv.W * cv.Cw);
            pix[l] = (oy << 16) | ox;
            pa[l] = A;
        } else {
            pa[l] = A + int64_t(rc) * lda;
        }
    }
    // binary: B rows staged like A.  planes: thread t stages word (2*kt + t/BN) of B row col0 + t%BN.
    const uint32_t* pb[NB];
    bool live_b[NB];
    const int bw_h = tid / BN, bw_r = tid % BN;
    if (PLANES) {
        live_b[0] = col0 + bw_r < N;
        pb[0] = B + int64_t(min(col0 + bw_r, N - 1)) * ldb;
    } else {
#pragma unroll
        for (int l = 0; l < LOADS_B; ++l) {
            const int r = col0 + st_r + l * ST_ROWS;
            live_b[l] = r < N;
            pb[l] = B + int64_t(min(r, N - 1)) * ldb;
        }
    }

    uint4 ra[LOADS_A], rb[NB];
    uint32_t rbw = 0u;
    int cnt_a[LOADS_A], cnt_b[NB];
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) cnt_a[l] = 0;
#pragma unroll
    for (int l = 0; l < NB; ++l) cnt_b[l] = 0;

    // Checked load of an A quad in the planes layout: every plane word of the last K-word is masked.
    auto load_quad_planes = [&](int row, int quad) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        const int w0 = quad * 4;
        if (row < M && w0 < kwa) {                      // kwa is a multiple of 8: the quad is complete
            const uint32_t* p = A + int64_t(row) * lda + w0;
            v = VEC ? *reinterpret_cast<const uint4*>(p) : make_uint4(p[0], p[1], p[2], p[3]);
            if ((w0 >> 3) == kw - 1) { v.x &= tmask; v.y &= tmask; v.z &= tmask; v.w &= tmask; }
        }
        return v;
    };
    // conv: quad `quad` of a receptive field is 4 channel words of one tap; the load address is
    // clamped into the image and the choice between the loaded words, all-ones and zeros is made
    // at staging, so the loads themselves are unconditional.
    auto fetch_conv = [&](int quad) {
        const int w0 = min(quad * 4, kwa - 4);
        const int tap = w0 / cv.Cw, cw = w0 - tap * cv.Cw;
        const int ky = tap / cv.kw, kx = tap - ky * cv.kw;
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            const int y = (pix[l] >> 16) * cv.stride - cv.pad + ky;
            const int x = (pix[l] & 0xFFFF) * cv.stride - cv.pad + kx;
            const bool inside = y >= 0 && y < cv.H && x >= 0 && x < cv.W;
            const int yc = min(max(y, 0), cv.H - 1), xc = min(max(x, 0), cv.W - 1);
            ra[l] = *reinterpret_cast<const uint4*>(A + img_off[l] + uint32_t((yc * cv.W + xc) * cv.Cw + cw));
            fill_a[l] = (!live_a[l] || quad * 4 >= kwa) ? 2 : (inside ? 0 : 1);
        }
    };
    auto fetch = [&](int kt) {
        const int quad = kt * kMfmaKQ + st_q;
        if (CONV) {
            fetch_conv(quad);
            if (kt < n_full_ktiles) {
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l) rb[l] = load_quad_unchecked<VEC>(pb[l], quad);
            } else {
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l)
                    rb[l] = load_quad<VEC>(B, ldb, N, kw, tmask, col0 + st_r + l * ST_ROWS, quad);
            }
        } else if (kt < n_full_ktiles) {
#pragma unroll
            for (int l = 0; l < LOADS_A; ++l) ra[l] = load_quad_unchecked<VEC>(pa[l], quad);
            if (PLANES) {
                rbw = pb[0][2 * kt + bw_h];
            } else {
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l) rb[l] = load_quad_unchecked<VEC>(pb[l], quad);
            }
        } else {
#pragma unroll
            for (int l = 0; l < LOADS_A; ++l) {
                const int r = row0 + st_r + l * ST_ROWS;
                if (PLANES) ra[l] = load_quad_planes(r, quad);
                else ra[l] = load_quad<VEC>(A, lda, M, kw, tmask, r, quad);
            }
            if (PLANES) {
                const int w = 2 * kt + bw_h;
                rbw = w < kw ? pb[0][w] : 0u;
                if (w == kw - 1) rbw &= tmask;
            } else {
#pragma unroll
                for (int l = 0; l < LOADS_B; ++l)
                    rb[l] = load_quad<VEC>(B, ldb, N, kw, tmask, col0 + st_r + l * ST_ROWS, quad);
            }
        }
    };
    // Writes the fetched words to LDS and adds their set bits to this thread's row sums.
    auto stage = [&](int buf) {
#pragma unroll
        for (int l = 0; l < LOADS_A; ++l) {
            // Rows beyond the matrix hold a copy of its last row (clamped load): their sums and
            // outputs are computed and never stored, so nothing has to be zeroed here.
            uint4 v = ra[l];
            if (CONV) {
                const bool keep = fill_a[l] == 0;
                const uint32_t fill = fill_a[l] == 1 ? ~0u : 0u;
                v = make_uint4(keep ? ra[l].x : fill, keep ? ra[l].y : fill, keep ? ra[l].z : fill,
                               keep ? ra[l].w : fill);
            }
            cnt_a[l] += PLANES ? popc4_weighted(v, 4 * (st_q & 1)) : popc4(v);
            lds_a[buf][st_q * PLANE_A + st_r + l * ST_ROWS] = v;
        }
        if (PLANES) {
            lds_bw[buf][bw_h * BN + bw_r] = rbw;
        } else {
#pragma unroll
            for (int l = 0; l < LOADS_B; ++l) {
                const uint4 v = rb[l];
                cnt_b[l] += popc4(v);
                lds_b[buf][st_q * PLANE_B + st_r + l * ST_ROWS] = v;
            }
        }
    };

    v16f acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    if (FUSED) {
        // No result exceeds lim in magnitude, so clamping a threshold to [-lim, lim] changes no output
        // bit and keeps the bounds the epilogue derives from it inside int32 for any caller-given value.
        const int lim = (PLANES ? 255 * K : K) + 1;
        if (tid < BN) thr_s[tid] = col0 + tid < N ? max(-lim, min(lim, bn.thr[col0 + tid])) : 0;
        if (tid < BN / 32) flip_s[tid] = col0 + 32 * tid < N ? bn.flip_bits[(col0 >> 5) + tid] : 0u;
    }
    if (n_ktiles > 0) {
        fetch(0);
        stage(0);
    }
    __syncthreads();

    constexpr int kScaleOne = 0x7f7f7f7f;      // E8M0 exponent 127 = scale 1.0 in every byte

    for (int kt = 0; kt < n_ktiles; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < n_ktiles) fetch(kt + 1);

        v8i fb[WN];
        if (PLANES) {
#pragma unroll
            for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(lds_bw[buf][fh * BN + wn * 32 * WN + j * 32 + fr]);
        }
        // The lane's 8 words are quads 2*fh and 2*fh+1 of its tile row; each quad feeds 4 steps.
#pragma unroll
        for (int hq = 0; hq < 2; ++hq) {
            uint4 aw[WM], bw[WN];
#pragma unroll
            for (int i = 0; i < WM; ++i) aw[i] = lds_a[buf][(2 * fh + hq) * PLANE_A + wm * 32 * WM + i * 32 + fr];
            if (!PLANES) {
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    bw[j] = lds_b[buf][(2 * fh + hq) * PLANE_B + wn * 32 * WN + j * 32 + fr];
            }
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                v8i fa[WM];
#pragma unroll
                for (int i = 0; i < WM; ++i) fa[i] = widen_fp4_a(quad_word(aw[i], s));
                if (!PLANES) {
#pragma unroll
                    for (int j = 0; j < WN; ++j) fb[j] = widen_fp4_b(quad_word(bw[j], s));
                }
                // planes: this step is plane 4*hq + s, weight 2^(4*hq + s) through the A block scale.
                // Without planes both block scales are 1: literal zero scale operands make the
                // compiler emit the plain v_mfma_f32_32x32x64_f8f6f4 (unit scale, half the encoding
                // size and no scale-register reads) instead of the scaled pair.
                const int scale_a = PLANES ? kScaleOne + (4 * hq + s) * 0x01010101 : 0;
                constexpr int scale_b = PLANES ? kScaleOne : 0;
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) {
                        if (BITS)
                            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                fb[j], fa[i], acc[i][j], 4 /* fp4 */, 4 /* fp4 */, 0, 0, 0, 0);
                        else
                            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(
                                fa[i], fb[j], acc[i][j], 4 /* A: fp4 */, 4 /* B: fp4 */, 0, scale_a, 0, scale_b);
                    }
            }
        }

        // Ordering pin: without it the compiler hoists the staging of the next tile (and with it
        // the wait for the global loads issued at the top of this iteration) above the MFMA steps,
        // which exposes the whole memory latency every iteration.  The empty asm "uses" the
        // accumulators, so all MFMAs precede it, and clobbers memory, so the LDS stores follow it.
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int j = 0; j < WN; ++j) asm volatile("" : "+v"(acc[i][j]) : : "memory");

        if (kt + 1 < n_ktiles) stage(buf ^ 1);
        __syncthreads();
    }

    // Row sums: the kMfmaKQ threads that staged the quads of one row are neighbouring lanes.
    // pop_a / pop_b hold 2*popcount (binary) or the plain row sum of the 8-bit inputs (planes).
#pragma unroll
    for (int l = 0; l < LOADS_A; ++l) {
        int c = cnt_a[l];
        c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);       // lane ^ 1
        c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);       // lane ^ 2
        if (st_q == 0) {
            pop_a[st_r + l * ST_ROWS] = PLANES ? c : 2 * c;
            if (FUSED) pop_af[st_r + l * ST_ROWS] = 0.5f * float(c);       // 2pa/4 (binary), rowsum/2 (planes)
        }
    }
#pragma unroll
    for (int l = 0; l < LOADS_B; ++l) {
        int c = cnt_b[l];
        c += __builtin_amdgcn_update_dpp(0, c, 0xB1, 0xF, 0xF, true);
        c += __builtin_amdgcn_update_dpp(0, c, 0x4E, 0xF, 0xF, true);
        if (st_q == 0) {
            pop_b[st_r + l * ST_ROWS] = 2 * c;
            if (BITS) colfix_s[st_r + l * ST_ROWS] = fold_column_term(thr_s[st_r + l * ST_ROWS], K, 2 * c);
        }
    }
    __syncthreads();

    if constexpr (BITS)
        mfma_epilogue_bits<WM, WN>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, colfix_s, bn, M, N, K, row0, col0, wm, wn,
                                   fr, fh);
    else
        mfma_epilogue<WM, WN, FUSED, PLANES>(acc, pop_a, pop_af, pop_b, thr_s, flip_s, C, ldc, bn, M, N, K, row0, col0,
                                             wm, wn, fr, fh);
}

template <int WM, bool FUSED, bool PLANES, bool CONV>
static int launch_mfma(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc,
                       int64_t M, int64_t N, int64_t K, BnSignArgs bn, ConvArgs cv, void* stream) {
    constexpr int WN = 2;
    const int64_t tiles_m = ceil_div(M, 64 * WM), tiles_n = ceil_div(N, 64 * WN);
    if (tiles_m * tiles_n > kMaxDim) return BNN_ERR_UNSUPPORTED;
    // The planes kernel reads B one word at a time, so only A's alignment matters there; the conv
    // kernel always reads whole 16-byte channel quads of A (its caller has checked that it can).
    const bool vec_a = CONV || (aligned_to(A, 16) && lda % 4 == 0);
    const bool vec = vec_a && (PLANES || (aligned_to(B, 16) && ldb % 4 == 0));
    const dim3 grid{unsigned(tiles_m * tiles_n)};
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (vec)
        hipLaunchKernelGGL((xnor_gemm_mfma_kernel<WM, WN, true, FUSED, PLANES, CONV>), grid, dim3(256), 0, s, A,
                           lda, B, ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn, cv);
    else
        hipLaunchKernelGGL((xnor_gemm_mfma_kernel<WM, WN, false, FUSED, PLANES, CONV>), grid, dim3(256), 0, s, A,
                           lda, B, ldb, C, ldc, int(M), int(N), int(K), int(tiles_m), int(tiles_n), bn, cv);
    return check_launch();
}

// Entry points used by the dispatchers.  The callers have validated the arguments.
bool mfma_path_supports(int64_t K) { return K <= kMfmaMaxAcc; }
bool mfma_planes_path_supports(int64_t K) { return 255 * K < kMfmaMaxAcc; }

int launch_xnor_gemm_mfma(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                          int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    return launch_mfma<4, false, false, false>(A, lda, B, ldb, C, ldc, M, N, K, BnSignArgs{}, ConvArgs{}, stream);
}

int launch_xnor_gemm_mfma_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    return launch_mfma<4, true, false, false>(A, lda, B, ldb, nullptr, 0, M, N, K, bn, ConvArgs{}, stream);
}

// 128 x 128 tiles (2 x 2 blocks per wavefront, 3 workgroups per compute unit): more, smaller
// workgroups for products whose K is short or whose 256 x 128 grid would leave units idle.  Grids
// of fewer than 256 such tiles take 64 x 128 tiles (1 x 2 blocks per wavefront) instead: with so few
// workgroups every one of them waits on its own K-tile loads, and twice as many share that wait
// (256 x 1024 x 8192 fused: 17.3 -> 13.0 us, 512 x 4096 x 4096: 10.3 -> 8.2 us).
static bool wants_half_tiles(int64_t M, int64_t N) { return ceil_div(M, 128) * ceil_div(N, 128) < 256; }

int launch_xnor_gemm_mfma128(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int32_t* C,
                             int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    if (wants_half_tiles(M, N))
        return launch_mfma<1, false, false, false>(A, lda, B, ldb, C, ldc, M, N, K, BnSignArgs{}, ConvArgs{}, stream);
    return launch_mfma<2, false, false, false>(A, lda, B, ldb, C, ldc, M, N, K, BnSignArgs{}, ConvArgs{}, stream);
}

int launch_xnor_gemm_mfma128_fused(const uint32_t* A, int64_t lda, const uint32_t* B, int64_t ldb, int64_t M,
                                   int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    if (wants_half_tiles(M, N))
        return launch_mfma<1, true, false, false>(A, lda, B, ldb, nullptr, 0, M, N, K, bn, ConvArgs{}, stream);
    return launch_mfma<2, true, false, false>(A, lda, B, ldb, nullptr, 0, M, N, K, bn, ConvArgs{}, stream);
}

int launch_bitplane_gemm_mfma(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int32_t* C,
                              int64_t ldc, int64_t M, int64_t N, int64_t K, void* stream) {
    return launch_mfma<4, false, true, false>(Xp, ldx, B, ldb, C, ldc, M, N, K, BnSignArgs{}, ConvArgs{}, stream);
}

int launch_bitplane_gemm_mfma_fused(const uint32_t* Xp, int64_t ldx, const uint32_t* B, int64_t ldb, int64_t M,
                                    int64_t N, int64_t K, BnSignArgs bn, void* stream) {
    return launch_mfma<4, true, true, false>(Xp, ldx, B, ldb, nullptr, 0, M, N, K, bn, ConvArgs{}, stream);
}

// Implicit-GEMM convolution: `in` is the packed NHWC input, B the packed filters [N][kh*kw*Cw].
// The conv kernel reads A in unaligned-tolerant fashion only through 16-byte quads, so the
// caller guarantees in is 16-byte aligned and Cw % 4 == 0.
// Tile choice as for the plain product: 256 x 128 when that grid fills the chip's 512 workgroup
// slots, else 128 x 128 (three workgroups per compute unit).
static bool conv_wants_small_tiles(int64_t M, int64_t N) { return ceil_div(M, 256) * ceil_div(N, 128) < 512; }

// Short receptive fields (K <= 1152: 3 x 3 over 128 channels) go to the conv mode of the short-K
// organisation (xnor_gemm_mfma_shortk.hip).
bool conv_shortk_supports(const uint32_t* B, int64_t ldb, int64_t K);
int launch_conv_mfma_shortk(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                            int64_t N, int64_t K, ConvArgs cv, void* stream);
int launch_conv_mfma_shortk_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N,
                                  int64_t K, BnSignArgs bn, ConvArgs cv, void* stream);

// "Same" convolutions whose tiles are whole image rows or whole images keep their input patch in
// LDS (conv_patch.hip); its launchers return BNN_ERR_UNSUPPORTED for every other geometry.
int launch_conv_patch(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                      int64_t N, int64_t K, ConvArgs cv, void* stream);
int launch_conv_patch_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                            BnSignArgs bn, ConvArgs cv, void* stream);

int launch_conv_mfma(const uint32_t* in, const uint32_t* B, int64_t ldb, int32_t* C, int64_t ldc, int64_t M,
                     int64_t N, int64_t K, ConvArgs cv, void* stream) {
    const int st = launch_conv_patch(in, B, ldb, C, ldc, M, N, K, cv, stream);
    if (st != BNN_ERR_UNSUPPORTED) return st;
    if (cv.Cw % 4 != 0) return BNN_ERR_UNSUPPORTED;     // the gathering loaders move whole 16-byte channel quads
    if (conv_shortk_supports(B, ldb, K)) return launch_conv_mfma_shortk(in, B, ldb, C, ldc, M, N, K, cv, stream);
    if (conv_wants_small_tiles(M, N))
        return launch_mfma<2, false, false, true>(in, 0, B, ldb, C, ldc, M, N, K, BnSignArgs{}, cv, stream);
    return launch_mfma<4, false, false, true>(in, 0, B, ldb, C, ldc, M, N, K, BnSignArgs{}, cv, stream);
}

int launch_conv_mfma_fused(const uint32_t* in, const uint32_t* B, int64_t ldb, int64_t M, int64_t N, int64_t K,
                           BnSignArgs bn, ConvArgs cv, void* stream) {
    const int st = launch_conv_patch_fused(in, B, ldb, M, N, K, bn, cv, stream);
    if (st != BNN_ERR_UNSUPPORTED) return st;
    if (cv.Cw % 4 != 0) return BNN_ERR_UNSUPPORTED;
    if (conv_shortk_supports(B, ldb, K)) return launch_conv_mfma_shortk_fused(in, B, ldb, M, N, K, bn, cv, stream);
    if (conv_wants_small_tiles(M, N))
        return launch_mfma<2, true, false, true>(in, 0, B, ldb, nullptr, 0, M, N, K, bn, cv, stream);
    return launch_mfma<4, true, false, true>(in, 0, B, ldb, nullptr, 0, M, N, K, bn, cv, stream);
}

}  // namespace bnn
