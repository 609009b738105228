/*
 * CPU oracle for the binarized-network forward hot path.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * obviously-correct CPU statement of what the GPU library must compute, and it
 * shares no code, header, table or helper with the HIP path.  Only tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it.
 *
 * Every routine works on literal +1/-1 values held in int8 (no bit tricks in
 * the arithmetic) and follows the paper by Courbariaux, Hubara, Soudry,
 * El-Yaniv and Bengio, "Binarized Neural Networks":
 *
 *   oracle_sign          Eq. (1): Sign(x) = +1 if x >= 0, -1 otherwise.
 *   oracle_matmul_pm1    Alg. 1 forward / Alg. 4: s_k = a^b_{k-1} W^b_k as a
 *                        literal integer multiply-add (the semantics of the
 *                        "baseline kernel" of Sec. 4, whose output the XNOR
 *                        kernel must equal on +-1 inputs).
 *   oracle_bn_float      Alg. 4: BatchNorm(a_k, theta_k) with running
 *                        statistics (the vanilla BatchNorm the paper cites),
 *                        in float32 with a fixed evaluation order.
 *   oracle_bn_sign       Alg. 4: a^b_k = Sign(BatchNorm(a_k, theta_k)).
 *   oracle_pack_bits /   Sec. 4: 32 binary variables concatenated into one
 *   oracle_unpack_bits   32-bit word (declared convention: bit=1 <=> +1,
 *                        element k in word k/32 at bit k%32, pad bits 0).
 *   oracle_conv_direct   Sec. 3.3 / Alg. 1 applied to a 2-D convolution:
 *                        direct sum over taps and channels, out-of-image
 *                        inputs read as +1 (zero padding through Sign(0)=+1).
 *   oracle_im2col        the definitional lowering of that convolution to a
 *                        matrix whose row m holds the receptive field of
 *                        output pixel m, K index = (ky*kw + kx)*Cin + ci.
 *   oracle_maxpool2d     plain window maximum of int32 pre-activations (the pooling the
 *                        paper's ConvNets apply between a convolution and its BatchNorm).
 *   oracle_first_layer_bitplanes
 *                        Alg. 4 step 1 / Eq. (4) of Sec. 1.6: 8-bit inputs as
 *                        sum_n 2^(n-1) <x^n, w^b>.
 *
 * Parity status: every function here is pinned by tests that run without a
 * GPU (sign table from Eq. (1); brute-force popcount identity; closed forms
 * incl. Sylvester-Hadamard; library matmul / conv2d / batch_norm / packbits).
 * Nothing is "parity unpinned".
 *
 * Build: gcc -O3 -fopenmp -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <math.h>
#include <stdint.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. (1).  IEEE comparison: +0.0 and -0.0 are both >= 0 (-> +1); NaN is not
 * >= 0 and falls in the "otherwise" branch (-> -1). */
static int8_t sign_f32(float x)
{
    return (x >= 0.0f) ? (int8_t)1 : (int8_t)-1;
}

void oracle_sign(const float *x, int64_t n, int8_t *out)
{
    for (int64_t i = 0; i < n; ++i)
        out[i] = sign_f32(x[i]);
}

/* C[m][n] = sum_k A[m][k] * Bm[k][n]; A is [M][K], Bm is the math layout
 * [K][N] (s = a W), all values +1/-1.  Loop order m,k,n so the inner loop is a
 * plain vectorisable axpy; no reordering beyond that. */
void oracle_matmul_pm1(const int8_t *A, const int8_t *Bm, int32_t *C,
                       int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int32_t *c = C + m * N;
        for (int64_t n = 0; n < N; ++n)
            c[n] = 0;
        for (int64_t k = 0; k < K; ++k) {
            const int32_t a = A[m * K + k];
            const int8_t *b = Bm + k * N;
            for (int64_t n = 0; n < N; ++n)
                c[n] += a * (int32_t)b[n];
        }
    }
}

/* Inference BatchNorm of one pre-activation, float32, no fused multiply-add:
 *   inv  = 1 / sqrt(var + eps)
 *   xhat = (s - mean) * inv
 *   y    = fl(fl(gamma * xhat) + beta)                                      */
static float bn_one(float s, float gamma, float beta, float mean, float var,
                    float eps)
{
    volatile float denom = sqrtf(var + eps);
    volatile float inv = 1.0f / denom;
    volatile float centred = s - mean;
    volatile float xhat = centred * inv;
    volatile float scaled = gamma * xhat;
    volatile float y = scaled + beta;
    return y;
}

/* Y[m][n] = BatchNorm_n(S[m][n]); channel = column n. */
void oracle_bn_float(const int32_t *S, int64_t M, int64_t N,
                     const float *gamma, const float *beta, const float *mean,
                     const float *var, float eps, float *Y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            Y[m * N + n] = bn_one((float)S[m * N + n], gamma[n], beta[n],
                                  mean[n], var[n], eps);
}

/* out[m][n] = Sign(BatchNorm_n(S[m][n])) as +1/-1. */
void oracle_bn_sign(const int32_t *S, int64_t M, int64_t N,
                    const float *gamma, const float *beta, const float *mean,
                    const float *var, float eps, int8_t *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n)
            out[m * N + n] = sign_f32(bn_one((float)S[m * N + n], gamma[n],
                                             beta[n], mean[n], var[n], eps));
}

/* 32 binary variables per 32-bit word.  words has ceil(cols/32) per row. */
void oracle_pack_bits(const int8_t *v, int64_t rows, int64_t cols,
                      uint32_t *words)
{
    const int64_t kw = (cols + 31) / 32;
    for (int64_t r = 0; r < rows; ++r) {
        for (int64_t w = 0; w < kw; ++w)
            words[r * kw + w] = 0u;
        for (int64_t k = 0; k < cols; ++k)
            if (v[r * cols + k] == 1)
                words[r * kw + k / 32] |= (uint32_t)1 << (k % 32);
    }
}

void oracle_unpack_bits(const uint32_t *words, int64_t rows, int64_t cols,
                        int8_t *v)
{
    const int64_t kw = (cols + 31) / 32;
    for (int64_t r = 0; r < rows; ++r)
        for (int64_t k = 0; k < cols; ++k)
            v[r * cols + k] =
                ((words[r * kw + k / 32] >> (k % 32)) & 1u) ? (int8_t)1
                                                            : (int8_t)-1;
}

/* Value of the +-1 input map at (b, y, x, ci); outside the image the value is
 * +1: the zero of zero-padding binarised by Eq. (1). */
static int32_t in_at(const int8_t *in, int64_t H, int64_t W, int64_t Cin,
                     int64_t b, int64_t y, int64_t x, int64_t ci)
{
    if (y < 0 || y >= H || x < 0 || x >= W)
        return 1;
    return in[((b * H + y) * W + x) * Cin + ci];
}

/* S[b][oy][ox][co] = sum_{ky,kx,ci} in(b, oy*stride+ky-pad, ox*stride+kx-pad, ci)
 *                                   * Wt[co][ky][kx][ci]
 * in is NHWC [B][H][W][Cin]; Wt is [Cout][kh][kw][Cin]; S is [B][Ho][Wo][Cout]
 * with Ho = (H + 2 pad - kh)/stride + 1 (same for Wo). */
void oracle_conv_direct(const int8_t *in, int64_t B, int64_t H, int64_t W,
                        int64_t Cin, const int8_t *Wt, int64_t Cout, int64_t kh,
                        int64_t kw, int64_t stride, int64_t pad, int32_t *S)
{
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1;
    const int64_t Wo = (W + 2 * pad - kw) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oy = 0; oy < Ho; ++oy)
            for (int64_t ox = 0; ox < Wo; ++ox)
                for (int64_t co = 0; co < Cout; ++co) {
                    int32_t acc = 0;
                    for (int64_t ky = 0; ky < kh; ++ky)
                        for (int64_t kx = 0; kx < kw; ++kx)
                            for (int64_t ci = 0; ci < Cin; ++ci)
                                acc += in_at(in, H, W, Cin, b,
                                             oy * stride + ky - pad,
                                             ox * stride + kx - pad, ci) *
                                       (int32_t)Wt[((co * kh + ky) * kw + kx) * Cin + ci];
                    S[((b * Ho + oy) * Wo + ox) * Cout + co] = acc;
                }
}

/* cols[(b*Ho+oy)*Wo+ox][(ky*kw+kx)*Cin+ci] = in(b, oy*stride+ky-pad, ox*stride+kx-pad, ci) */
void oracle_im2col(const int8_t *in, int64_t B, int64_t H, int64_t W,
                   int64_t Cin, int64_t kh, int64_t kw, int64_t stride,
                   int64_t pad, int8_t *cols)
{
    const int64_t Ho = (H + 2 * pad - kh) / stride + 1;
    const int64_t Wo = (W + 2 * pad - kw) / stride + 1;
    const int64_t K = kh * kw * Cin;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t oy = 0; oy < Ho; ++oy)
            for (int64_t ox = 0; ox < Wo; ++ox) {
                int8_t *row = cols + ((b * Ho + oy) * Wo + ox) * K;
                for (int64_t ky = 0; ky < kh; ++ky)
                    for (int64_t kx = 0; kx < kw; ++kx)
                        for (int64_t ci = 0; ci < Cin; ++ci)
                            row[(ky * kw + kx) * Cin + ci] = (int8_t)in_at(
                                in, H, W, Cin, b, oy * stride + ky - pad,
                                ox * stride + kx - pad, ci);
            }
}

/* Max pooling of the integer pre-activations.  Sec. 2.2 only says its ConvNet has the
 * architecture of the BinaryConnect network it cites; that every second convolution is
 * followed by 2x2 max pooling, placed between the convolution and its BatchNorm, is this
 * build's reading of that cited architecture (the paper prints neither):
 *   P[b][py][px][c] = max over (dy < ph, dx < pw) of S[b][py*stride+dy][px*stride+dx][c]
 * No padding; Hp = (H - ph)/stride + 1, Wp likewise. */
void oracle_maxpool2d(const int32_t *S, int64_t B, int64_t H, int64_t W, int64_t C,
                      int64_t ph, int64_t pw, int64_t stride, int32_t *P)
{
    const int64_t Hp = (H - ph) / stride + 1;
    const int64_t Wp = (W - pw) / stride + 1;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t py = 0; py < Hp; ++py)
            for (int64_t px = 0; px < Wp; ++px)
                for (int64_t c = 0; c < C; ++c) {
                    int32_t best = S[((b * H + py * stride) * W + px * stride) * C + c];
                    for (int64_t dy = 0; dy < ph; ++dy)
                        for (int64_t dx = 0; dx < pw; ++dx) {
                            const int32_t v =
                                S[((b * H + py * stride + dy) * W + px * stride + dx) * C + c];
                            if (v > best)
                                best = v;
                        }
                    P[((b * Hp + py) * Wp + px) * C + c] = best;
                }
}

/* First layer on 8-bit fixed-point inputs (Sec. 1.6, Alg. 4 step 1):
 *   s[m][n] = sum_{p=1..8} 2^(p-1) * sum_k x^p[m][k] * Wb[k][n]
 * where x^p[m][k] in {0,1} is bit p (1 = least significant) of X[m][k].
 * X is [M][K] uint8, Wb is [K][N] +-1.  Written plane by plane, exactly as
 * the algorithm states; equals the plain integer product sum_k X*W. */
void oracle_first_layer_bitplanes(const uint8_t *X, const int8_t *Wb,
                                  int32_t *S, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        int32_t *s = S + m * N;
        for (int64_t n = 0; n < N; ++n)
            s[n] = 0;
        for (int p = 1; p <= 8; ++p) {
            const int32_t weight = (int32_t)1 << (p - 1);
            for (int64_t k = 0; k < K; ++k) {
                const int32_t xbit = (X[m * K + k] >> (p - 1)) & 1;
                const int8_t *w = Wb + k * N;
                for (int64_t n = 0; n < N; ++n)
                    s[n] += weight * (xbit * (int32_t)w[n]);
            }
        }
    }
}
