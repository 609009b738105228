/*
 * bnn.h - C ABI of the MI355X (gfx950) library for the forward hot path of
 * Binarized Neural Networks (Courbariaux, Hubara, Soudry, El-Yaniv, Bengio).
 *
 * The path is the hidden-layer loop of Alg. 4 ("Running a BNN"):
 *     a_k   = XnorDotProduct(a^b_{k-1}, W^b_k)
 *     a^b_k = Sign(BatchNorm(a_k, theta_k))
 * on +-1 values concatenated 32 per 32-bit word (Sec. 4, Eq. (5)).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Packed rows: bit = 1 <=> +1, bit = 0 <=> -1.  Element k of a row lives in
 *    word k / 32 at bit k % 32 (least significant bit first).  A row of K
 *    elements occupies bnn_words_per_row(K) words; the unused high bits of its
 *    last word ("pad bits") are written as 0 by this library, and are ignored
 *    (masked) wherever this library reads packed operands.
 *  - Matrices are row-major with a leading dimension ("ld", counted in
 *    elements of the array's own type: floats, words, int32 or bytes).
 *  - Unless an argument is marked HOST, every pointer is a DEVICE pointer on
 *    the current HIP device, owned by the caller.  The library allocates
 *    nothing, keeps no pointer after returning, and never synchronises: work
 *    is enqueued on `stream` (a hipStream_t passed as void*; NULL = the
 *    default stream) and the caller orders it against its own work.
 *  - Inputs and outputs must not overlap.
 *  - Every function returns a bnn_status.  On any status other than BNN_OK no
 *    kernel was launched and no output was written.  A dimension of 0 for
 *    rows/M/N/B is a valid empty problem: BNN_OK, nothing launched.
 *  - Limits: every dimension < 2^31; K <= 2^31 - 32 for every product, so that
 *    |dot| <= K, the threshold K + 1 and the word count (K + 31) / 32 stay inside
 *    32-bit arithmetic (bnn_bn_fold alone accepts a range up to 2^31 - 2).
 */
#ifndef BNN_H
#define BNN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BNN_VERSION 100 /* 0.1.0 */

typedef enum bnn_status {
    BNN_OK = 0,
    BNN_ERR_INVALID_ARG = 1, /* null pointer, negative size, ld too small, K out of range */
    BNN_ERR_ALIGNMENT = 2,   /* pointer not aligned to its element type */
    BNN_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for */
    BNN_ERR_LAUNCH = 4       /* the HIP runtime refused the launch */
} bnn_status;

int bnn_version(void);
const char *bnn_status_string(int status);

/* ceil(K / 32): words in a packed row of K elements (Sec. 4: 32 binary
 * variables per 32-bit register).  Returns -1 if K < 0. */
int64_t bnn_words_per_row(int64_t K);

/*
 * Eq. (1) + Sec. 4 packing:  out[r][k/32] bit (k%32) = (x[r][k] >= 0).
 * The comparison is the IEEE one: +0.0, -0.0 -> 1; negative subnormals -> 0;
 * NaN -> 0.
 *   x     [rows][ld_x] float32, ld_x >= cols
 *   out   [rows][ld_out] uint32, ld_out >= ceil(cols/32); words
 *         [ceil(cols/32), ld_out) of each row are left untouched
 * Fast path when x is 16-byte aligned and ld_x % 4 == 0; any other layout
 * takes a slower element-wise path with the same result.
 */
int bnn_pack_sign(const float *x, int64_t rows, int64_t cols, int64_t ld_x,
                  uint32_t *out, int64_t ld_out, void *stream);

/*
 * Sec. 4, Eq. (5) over whole matrices (the XnorDotProduct of Alg. 4):
 *   C[m][n] = sum_{k<K} a[m][k] * b[n][k],  a, b in {-1,+1}
 *           = 2 * popcount(xnor(A[m], B[n]) over the K valid bits) - K
 * computed as K - 2 * sum_w popcount(A[m][w] ^ B[n][w]) with the pad bits of
 * both operands masked off, so their content never matters.
 *   A  [M][lda] packed rows of K bits (activations a^b)
 *   B  [N][ldb] packed rows of K bits: row n is output unit n's weight vector,
 *      i.e. B is the transpose of W^b in s = a W (both operands K-contiguous)
 *   C  [M][ldc] int32, ldc >= N
 * lda, ldb >= ceil(K/32).  Fast tiles need A, B 16-byte aligned with lda, ldb
 * multiples of 4; other layouts run a slower path with the same result.
 * K == 0 writes C = 0.
 */
int bnn_xnor_gemm(const uint32_t *A, int64_t lda, const uint32_t *B, int64_t ldb,
                  int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                  void *stream);

/* Same contract, with the kernel chosen by the caller (for tests and
 * profiling): 0 = automatic (what bnn_xnor_gemm does), 1 = one thread per
 * output, 2 = 128x128 LDS-tiled register-blocked XNOR-popcount kernel,
 * 3 = K-split kernel with wavefront reduction (skinny outputs), 4 = 64x64
 * tiled XNOR-popcount kernel, 5 = bits-in / matrix-engine-inside kernel (bits
 * widened to 4-bit floats in registers, MFMA, 256x128 tiles; needs
 * K <= 2^24, else BNN_ERR_UNSUPPORTED), 6 = the same with 128x128 tiles,
 * 7 = the same arithmetic organised for short K (a workgroup keeps its 128
 * columns of B in LDS and walks over several 128-row tiles of A; needs
 * 96 < K <= 1152, A and B 16-byte aligned, lda and ldb multiples of 4, else
 * BNN_ERR_UNSUPPORTED), 8 = kernel 5 as a tile walk (one workgroup per
 * resident slot walks over several 256x128 tiles, fetching the next tile's
 * first operands under the current tile's last products; needs more tiles
 * than slots, K a multiple of 512 with 1024 <= K <= 2^24, N a multiple of
 * 128, M >= 256, A and B 16-byte aligned, lda and ldb multiples of 4 below
 * 2^22, else BNN_ERR_UNSUPPORTED; what 0 picks when the last round of tiles
 * would fill only part of the chip), 9 = a kernel of the fused product
 * only (BNN_ERR_UNSUPPORTED here), 10 = the arithmetic of kernel 5 on 32x32
 * output tiles with K split over the four wavefronts of a workgroup and the
 * operands read from memory straight into the MFMA's registers (for small
 * outputs with a long K, such as fully connected layers at batch 256; needs
 * K a positive multiple of 128 up to 2^24, A and B 16-byte aligned, lda and
 * ldb multiples of 4, else BNN_ERR_UNSUPPORTED; what 0 picks, from K = 512
 * on, for outputs of at most 256 such tiles, at most 512 with K >= 2048 or
 * at most 1024 with K >= 4096).  Unknown ids give BNN_ERR_INVALID_ARG. */
int bnn_xnor_gemm_kernel(const uint32_t *A, int64_t lda, const uint32_t *B, int64_t ldb,
                         int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                         int kernel_id, void *stream);

/*
 * HOST function.  Folds Sign(BatchNorm(s)) of Alg. 4 (inference BatchNorm with
 * running statistics, evaluated in float32 as
 *     y = gamma * ((float(s) - mean) * (1 / sqrt(var + eps))) + beta,
 * every operation rounded separately) into one integer compare per channel:
 *     Sign(y(s)) = +1  <=>  (s >= thr[n]) XOR flip[n]     for all integer s in [-K, K].
 * The threshold is found by searching the float expression itself (which is
 * monotone in s), not by solving it algebraically, so the equivalence is exact
 * at rounding boundaries.  gamma < 0 reverses the inequality (flip = 1);
 * gamma == 0 gives a constant bit (thr = -K or K + 1).
 *   gamma, beta, mean, var  HOST [N] float32; all finite, var + eps > 0
 *   thr        HOST [N] int32, each in [-K, K + 1]
 *   flip_bits  HOST [ceil(N/32)] uint32, channel n at word n/32 bit n%32, pad bits 0
 * Non-finite parameters or var + eps <= 0 give BNN_ERR_INVALID_ARG.
 */
int bnn_bn_fold(const float *gamma, const float *beta, const float *mean,
                const float *var, float eps, int64_t N, int64_t K, int32_t *thr,
                uint32_t *flip_bits);

/*
 * Alg. 4, a^b_k = Sign(BatchNorm(a_k, theta_k)), on folded parameters, packed
 * for the next layer:
 *   out[m][n/32] bit (n%32) = (C[m][n] >= thr[n]) XOR flip[n]
 *   C    [M][ldc] int32, ldc >= N
 *   thr  [N] int32 (device), flip_bits [ceil(N/32)] uint32 (device), from bnn_bn_fold
 *        (any int32 is a valid threshold; pad bits of the last flip word must be 0)
 *   out  [M][ld_out] uint32, ld_out >= ceil(N/32); pad bits of the last word 0;
 *        words beyond ceil(N/32) untouched
 * Fast path when C and thr are 16-byte aligned and ldc % 4 == 0.
 */
int bnn_bn_sign_pack(const int32_t *C, int64_t ldc, int64_t M, int64_t N,
                     const int32_t *thr, const uint32_t *flip_bits, uint32_t *out,
                     int64_t ld_out, void *stream);

/*
 * One hidden layer of Alg. 4 in a single launch:
 *     a_k   = XnorDotProduct(a^b_{k-1}, W^b_k)
 *     a^b_k = Sign(BatchNorm(a_k, theta_k))
 * i.e. bnn_xnor_gemm followed by bnn_bn_sign_pack with the int32
 * pre-activations kept in registers (they never reach memory):
 *   out[m][n/32] bit (n%32) = (C[m][n] >= thr[n]) XOR flip[n],
 *   C[m][n] = K - 2 * sum_w popcount(A[m][w] ^ B[n][w]).
 * Arguments as in those two calls (A [M][lda], B [N][ldb] packed rows of K bits;
 * thr [N], flip_bits [ceil(N/32)] device arrays from bnn_bn_fold;
 * out [M][ld_out], ld_out >= ceil(N/32), pad bits 0, words beyond untouched).
 * The result is bit-identical to the two-call sequence for every int32 threshold.
 */
int bnn_xnor_gemm_bn_sign_pack(const uint32_t *A, int64_t lda, const uint32_t *B, int64_t ldb,
                               int64_t M, int64_t N, int64_t K, const int32_t *thr,
                               const uint32_t *flip_bits, uint32_t *out, int64_t ld_out,
                               void *stream);

/* Same contract with the kernel chosen by the caller: 0 = automatic, 2, 4, 5, 6, 7, 8 as
 * in bnn_xnor_gemm_kernel (the other kernels have no fused form), 9 = the arithmetic of
 * kernel 5 on 256x256 tiles with one wavefront per SIMD and one workgroup per compute
 * unit, which takes a strip of rows of one 256-column tile as 256-row tiles and at most
 * one 128-row tile (needs K a multiple of 512 with 2048 <= K <= 2^19, N a multiple of
 * 256 whose tile count N/256 divides the compute units, M / (compute units / (N/256))
 * >= 256, A and B 16-byte aligned, lda and ldb multiples of 4 below 2^22, out 8-byte
 * aligned, ld_out even, else BNN_ERR_UNSUPPORTED; what 0 picks for such products when
 * a strip has at least 512 rows or exactly 256), 10 as in bnn_xnor_gemm_kernel. */
int bnn_xnor_gemm_bn_sign_pack_kernel(const uint32_t *A, int64_t lda, const uint32_t *B, int64_t ldb,
                                      int64_t M, int64_t N, int64_t K, const int32_t *thr,
                                      const uint32_t *flip_bits, uint32_t *out, int64_t ld_out,
                                      int kernel_id, void *stream);

/*
 * First layer on 8-bit fixed-point inputs (Sec. 1.6; Alg. 4 step 1):
 *     a_1 = sum_{n=1..8} 2^(n-1) * <a_0^n, W^b_1>,   a_0^n in {0,1} the n-th bit plane.
 *
 * bnn_pack_bitplanes splits uint8 inputs into packed bit planes:
 *   out[r][8*w + p] bit j = bit p (p = 0 least significant, the paper's n = p+1) of x[r][32*w + j]
 *   x   [rows][ld_x] uint8, ld_x >= cols
 *   out [rows][ld_out] uint32, ld_out >= 8*ceil(cols/32); elements >= cols read as 0; words beyond
 *       8*ceil(cols/32) untouched.  Fast path when x is 4-byte aligned and ld_x % 4 == 0.
 *
 * bnn_bitplane_gemm:  C[m][n] = sum_k x[m][k] * w[n][k],  x in [0,255] given as bit planes (layout
 *   above, Xp [M][ldx], ldx >= 8*ceil(K/32)), w in {-1,+1} given as packed rows B [N][ldb] as in
 *   bnn_xnor_gemm; C [M][ldc] int32.  Computed plane by plane on the matrix engine with the plane
 *   weight 2^(n-1) as block scale while 255*K < 2^24 (the exact range of its accumulation); larger
 *   K is computed with and/popcount on the vector ALU (slow, exact).  255*K must fit int32
 *   (255*K <= 2^31 - 32), else BNN_ERR_INVALID_ARG.  Pad bits of the last K-word of either operand
 *   are ignored.
 *
 * bnn_bitplane_gemm_bn_sign_pack: the same product followed by Sign(BatchNorm(a_1, theta_1)) on
 *   folded thresholds (bnn_bn_fold with 255*K as the range argument), written as packed bits:
 *   out[m][n/32] bit (n%32) = (C[m][n] >= thr[n]) XOR flip[n]; out as in bnn_bn_sign_pack.
 */
int bnn_pack_bitplanes(const uint8_t *x, int64_t rows, int64_t cols, int64_t ld_x,
                       uint32_t *out, int64_t ld_out, void *stream);
int bnn_bitplane_gemm(const uint32_t *Xp, int64_t ldx, const uint32_t *B, int64_t ldb,
                      int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K, void *stream);
int bnn_bitplane_gemm_bn_sign_pack(const uint32_t *Xp, int64_t ldx, const uint32_t *B, int64_t ldb,
                                   int64_t M, int64_t N, int64_t K, const int32_t *thr,
                                   const uint32_t *flip_bits, uint32_t *out, int64_t ld_out,
                                   void *stream);

/*
 * Lowers a binary kh x kw convolution (3 x 3 in the paper's nets, Sec. 3.3) to
 * the matrix product above: row m = (b*Ho + oy)*Wo + ox of `out` holds the
 * receptive field of output pixel (b, oy, ox) as K = kh*kw*Cin bits,
 *   bit (ky*kw + kx)*Cin + ci = in(b, oy*stride + ky - pad, ox*stride + kx - pad, ci),
 * and taps that fall outside the image read as +1 (bit 1): zero padding
 * binarised by Eq. (1), Sign(0) = +1.  Ho = (H + 2*pad - kh)/stride + 1, same for Wo.
 *   in   packed NHWC [B][H][W][ceil(Cin/32)] uint32 (pad bits ignored)
 *   out  [B*Ho*Wo][ld_out] uint32, ld_out >= ceil(kh*kw*Cin/32); pad bits 0
 * Weights for the product are [Cout][kh][kw][Cin] packed along (ky,kx,ci).
 * Cin % 32 == 0 copies whole words; other Cin take a bit-gather path.
 * Requires kh, kw, stride >= 1, pad >= 0 and Ho, Wo >= 1.
 */
int bnn_conv_im2col_pack(const uint32_t *in, int64_t B, int64_t H, int64_t W,
                         int64_t Cin, int kh, int kw, int stride, int pad,
                         uint32_t *out, int64_t ld_out, void *stream);

/*
 * A whole binary convolution layer without the intermediate matrix (implicit GEMM): the
 * receptive fields described under bnn_conv_im2col_pack are taken straight from the packed NHWC
 * input - from a patch of it held on chip for same-size stride-1 convolutions, gathered by the
 * product's tile loader otherwise.
 *   S[(b*Ho + oy)*Wo + ox][co] = sum_{ky,kx,ci} in(b, oy*stride+ky-pad, ox*stride+kx-pad, ci) * Wt[co][ky][kx][ci]
 *   in   packed NHWC [B][H][W][Cin/32] uint32, out-of-image taps read as +1
 *   Wb   packed filters [Cout][ldw], row co = Wt[co] flattened as (ky, kx, ci), ldw >= kh*kw*Cin/32
 *   bnn_conv_xnor:          S [B*Ho*Wo][lds] int32, lds >= Cout
 *   bnn_conv_bn_sign_pack:  out [B*Ho*Wo][ld_out] packed bits = (S >= thr[co]) XOR flip[co]
 *                           (= packed NHWC input of the next layer), thr/flip from bnn_bn_fold
 * Bit-identical to bnn_conv_im2col_pack followed by bnn_xnor_gemm (and bnn_bn_sign_pack).
 * Receptive fields of more than 2^24 bits (beyond the matrix engine's exact range) take a slow, exact
 * xor/popcount kernel for any geometry with Cin % 32 == 0.
 * Requires H, W, pad, Ho, Wo <= 32767, an input of fewer than 2^32 words, and either
 *   Cin % 128 == 0 with `in` 16-byte aligned (any kh, kw, stride, pad), or
 *   Cin % 32 == 0 on a same-size stride-1 layer (kh = kw = 2*pad + 1) whose image rows fit the kernel's
 *   128-pixel tiles (W divides 128; H a multiple of 128/W or the reverse), with kh*kw*Cin <= 2560 and
 *   Wb 16-byte aligned, ldw % 4 == 0 (e.g. the 64-channel 3 x 3 layers of the half-width net of Sec. 2.3);
 * otherwise BNN_ERR_UNSUPPORTED (use the im2col path).
 */
int bnn_conv_xnor(const uint32_t *in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                  const uint32_t *Wb, int64_t ldw, int64_t Cout, int kh, int kw, int stride, int pad,
                  int32_t *S, int64_t lds, void *stream);
int bnn_conv_bn_sign_pack(const uint32_t *in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                          const uint32_t *Wb, int64_t ldw, int64_t Cout, int kh, int kw, int stride,
                          int pad, const int32_t *thr, const uint32_t *flip_bits, uint32_t *out,
                          int64_t ld_out, void *stream);

/*
 * The pooled layer of the paper's ConvNets in one launch: convolution, pool x pool max pooling
 * (stride pool) of the pre-activations, BatchNorm, Sign (Alg. 4 for the last two).  Sec. 2.2 only says
 * that its ConvNet has the architecture of the BinaryConnect network it cites; that pooling sits between
 * a convolution and its BatchNorm is this library's reading of that cited architecture, not a statement
 * the paper prints.
 *   out [B*(Ho/pool)*(Wo/pool)][ld_out] packed bits, the packed NHWC input of the next layer;
 *   every other argument as in bnn_conv_bn_sign_pack.
 * Bit-identical to bnn_conv_bn_sign_pack followed by bnn_maxpool_bits (see there for why pooling
 * the output bits equals pooling the pre-activations).  Only pool = 2 on same-size stride-1
 * convolutions whose tiles hold whole, even numbers of image rows is taken (even H and W; W a power
 * of two up to 16, or 32 or 64; the requirements of bnn_conv_bn_sign_pack); anything else returns
 * BNN_ERR_UNSUPPORTED before any launch: use the two calls then.
 */
int bnn_conv_pool_bn_sign_pack(const uint32_t *in, int64_t B, int64_t H, int64_t W, int64_t Cin,
                               const uint32_t *Wb, int64_t ldw, int64_t Cout, int kh, int kw, int stride,
                               int pad, int pool, const int32_t *thr, const uint32_t *flip_bits,
                               uint32_t *out, int64_t ld_out, void *stream);

/*
 * Max pooling for binarized layers.  In the architecture Sec. 2.2 refers to (the cited BinaryConnect
 * ConvNet, as this library reads it) the pre-activations are pooled between a convolution and its
 * BatchNorm + Sign; since Sign(BatchNorm(.)) is monotone per channel, the bit
 * of the pooled pre-activation is the OR of the window's bits where the channel's folded flip
 * bit is 0 and their AND where it is 1, so pooling runs on the packed output of the fused layer:
 *   out[b][py][px][c] = OR / AND over dy < ph, dx < pw of in[b][py*stride+dy][px*stride+dx][c]
 *   in  packed NHWC [B][H][W][ceil(C/32)], out packed NHWC [B][Hp][Wp][ceil(C/32)],
 *   Hp = (H - ph)/stride + 1, Wp = (W - pw)/stride + 1 (no padding)
 *   flip_bits [ceil(C/32)] device words from bnn_bn_fold, or NULL for OR on every channel.
 * Pad bits of `in` pass through the same operations (zero stays zero under OR).
 */
int bnn_maxpool_bits(const uint32_t *in, int64_t B, int64_t H, int64_t W, int64_t C, int ph, int pw,
                     int stride, const uint32_t *flip_bits, uint32_t *out, void *stream);

/*
 * The competing dense-engine variant of the same product (the role the vendor
 * GEMM plays in Sec. 4 / Fig. 3): +-1 stored one per int8, multiplied on the
 * int8 MFMA units with int32 accumulation.
 *   C[m][n] = sum_k A[m][k] * B[n][k]
 *   A [M][lda] int8, B [N][ldb] int8 (row n = weights of output n), C [M][ldc] int32
 * Exact for any int8 contents with |sum| < 2^31.  Requires A, B 16-byte
 * aligned and lda, ldb multiples of 16 (else BNN_ERR_ALIGNMENT); K need not be.
 */
int bnn_gemm_i8_mfma(const int8_t *A, int64_t lda, const int8_t *B, int64_t ldb,
                     int32_t *C, int64_t ldc, int64_t M, int64_t N, int64_t K,
                     void *stream);

/* Expands packed rows to one int8 (+1 / -1) per element, the operand format of
 * bnn_gemm_i8_mfma: out[r][k] = bit k of in[r] ? +1 : -1 for k < K, and 0 for
 * K <= k < ld_out (so padded columns add nothing to a product).
 *   in [rows][ld_in] uint32, out [rows][ld_out] int8, ld_out >= K.
 * out is written four bytes at a time: it must be 4-byte aligned and ld_out a
 * multiple of 4, else BNN_ERR_ALIGNMENT (bnn_gemm_i8_mfma wants 16 for both anyway). */
int bnn_unpack_i8(const uint32_t *in, int64_t ld_in, int64_t rows, int64_t K,
                  int8_t *out, int64_t ld_out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BNN_H */
