// A caller of the C ABI that is not Python: one hidden layer of Alg. 4 (Sign + pack, XnorDotProduct,
// Sign(BatchNorm)) on ragged sizes, through include/bnn.h alone, with device memory from the HIP
// runtime.  Checks, on the host:
//   - bnn_xnor_gemm against the literal +-1 product of the Sign-binarized inputs (Eq. (1), Sec. 4);
//   - bnn_bn_sign_pack on its result against (C >= thr) XOR flip with the folded parameters;
//   - bnn_xnor_gemm_bn_sign_pack against that two-call sequence, word for word.
// Prints "c_abi ok" and returns 0, or says what differed and returns 1.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "bnn.h"

#define HIP_OK(call)                                                                      \
    do {                                                                                  \
        hipError_t e_ = (call);                                                           \
        if (e_ != hipSuccess) {                                                           \
            std::fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)
#define BNN_OK_OR_FAIL(call)                                                              \
    do {                                                                                  \
        int s_ = (call);                                                                  \
        if (s_ != BNN_OK) {                                                               \
            std::fprintf(stderr, "%s returned %d (%s)\n", #call, s_, bnn_status_string(s_)); \
            return 1;                                                                     \
        }                                                                                 \
    } while (0)

// xorshift: the draws only have to be the same on both sides of the comparison
static uint32_t next(uint32_t& s) {
    s ^= s << 13;
    s ^= s >> 17;
    s ^= s << 5;
    return s;
}

int main() {
    const int64_t M = 70, N = 45, K = 203;
    const int64_t kw = bnn_words_per_row(K), nw = bnn_words_per_row(N);
    uint32_t seed = 160202830u;
    std::vector<float> a(M * K), w(N * K);
    for (auto& v : a) v = float(int(next(seed) % 2001) - 1000) / 1000.0f;          // includes exact zeros
    for (auto& v : w) v = float(int(next(seed) % 2001) - 1000) / 1000.0f;
    std::vector<float> gamma(N), beta(N), mean(N), var(N);
    for (int64_t n = 0; n < N; ++n) {
        gamma[n] = (n % 7 == 3 ? -1.0f : 1.0f) * (0.5f + float(next(seed) % 100) / 100.0f);
        beta[n] = float(int(next(seed) % 200) - 100) / 100.0f;
        mean[n] = float(int(next(seed) % 40) - 20);
        var[n] = float(K) * (0.5f + float(next(seed) % 100) / 100.0f);
    }
    std::vector<int32_t> thr(N);
    std::vector<uint32_t> flip(nw);
    BNN_OK_OR_FAIL(bnn_bn_fold(gamma.data(), beta.data(), mean.data(), var.data(), 1e-4f, N, K, thr.data(), flip.data()));

    float *d_a, *d_w;
    uint32_t *d_ab, *d_wb, *d_flip, *d_bits, *d_fused;
    int32_t *d_c, *d_thr;
    HIP_OK(hipMalloc(&d_a, a.size() * 4));
    HIP_OK(hipMalloc(&d_w, w.size() * 4));
    HIP_OK(hipMalloc(&d_ab, M * kw * 4));
    HIP_OK(hipMalloc(&d_wb, N * kw * 4));
    HIP_OK(hipMalloc(&d_c, M * N * 4));
    HIP_OK(hipMalloc(&d_thr, N * 4));
    HIP_OK(hipMalloc(&d_flip, nw * 4));
    HIP_OK(hipMalloc(&d_bits, M * nw * 4));
    HIP_OK(hipMalloc(&d_fused, M * nw * 4));
    HIP_OK(hipMemcpy(d_a, a.data(), a.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_w, w.data(), w.size() * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_thr, thr.data(), N * 4, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_flip, flip.data(), nw * 4, hipMemcpyHostToDevice));

    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));
    BNN_OK_OR_FAIL(bnn_pack_sign(d_a, M, K, K, d_ab, kw, stream));
    BNN_OK_OR_FAIL(bnn_pack_sign(d_w, N, K, K, d_wb, kw, stream));
    BNN_OK_OR_FAIL(bnn_xnor_gemm(d_ab, kw, d_wb, kw, d_c, N, M, N, K, stream));
    BNN_OK_OR_FAIL(bnn_bn_sign_pack(d_c, N, M, N, d_thr, d_flip, d_bits, nw, stream));
    BNN_OK_OR_FAIL(bnn_xnor_gemm_bn_sign_pack(d_ab, kw, d_wb, kw, M, N, K, d_thr, d_flip, d_fused, nw, stream));
    HIP_OK(hipStreamSynchronize(stream));

    std::vector<int32_t> c(M * N);
    std::vector<uint32_t> bits(M * nw), fused(M * nw);
    HIP_OK(hipMemcpy(c.data(), d_c, c.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(bits.data(), d_bits, bits.size() * 4, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(fused.data(), d_fused, fused.size() * 4, hipMemcpyDeviceToHost));

    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int dot = 0;
            for (int64_t k = 0; k < K; ++k) dot += (a[m * K + k] >= 0.0f ? 1 : -1) * (w[n * K + k] >= 0.0f ? 1 : -1);
            if (c[m * N + n] != dot) {
                std::fprintf(stderr, "C[%ld][%ld] = %d, literal product %d\n", long(m), long(n), c[m * N + n], dot);
                return 1;
            }
            const uint32_t want = uint32_t(dot >= thr[n]) ^ ((flip[n / 32] >> (n % 32)) & 1u);
            const uint32_t got = (bits[m * nw + n / 32] >> (n % 32)) & 1u;
            if (got != want) {
                std::fprintf(stderr, "bit[%ld][%ld] = %u, want %u\n", long(m), long(n), got, want);
                return 1;
            }
        }
    for (size_t i = 0; i < bits.size(); ++i)
        if (bits[i] != fused[i]) {
            std::fprintf(stderr, "fused word %zu = %08x, two-call sequence %08x\n", i, fused[i], bits[i]);
            return 1;
        }
    for (int64_t m = 0; m < M; ++m)                       // pad bits of the last word are zero
        if (N % 32 && (bits[m * nw + nw - 1] >> (N % 32)) != 0u) {
            std::fprintf(stderr, "pad bits set in row %ld\n", long(m));
            return 1;
        }
    std::printf("c_abi ok: %ld x %ld x %ld hidden layer through the C ABI (version %d)\n", long(M), long(N), long(K),
                bnn_version());
    return 0;
}
