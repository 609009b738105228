// bnn_bn_fold (HOST): folds Sign(BatchNorm(s)) of Alg. 4 into one integer
// compare per channel.
//
// For a fixed channel the float32 expression
//     y(s) = gamma * ((float(s) - mean) * (1 / sqrt(var + eps))) + beta
// is a chain of correctly rounded operations, each monotone in its s-dependent
// operand (int -> float conversion, subtracting a constant, multiplying by a
// positive constant, multiplying by gamma, adding a constant).  So the set
// {s : y(s) >= 0} is an up-set (gamma > 0), a down-set (gamma < 0) or
// everything / nothing, and its edge is found by bisection on the expression
// itself.  Solving for the threshold algebraically would be off by one at
// rounding boundaries.
//
// This file must be compiled without floating-point contraction.
#include <cmath>
#include <cstdint>

#include "bnn.h"

namespace {

struct Channel {
    float gamma, beta, mean, inv;
};

// Each step through a volatile so that no compiler fuses or reorders them.
inline bool bn_nonneg(const Channel& c, int64_t s) {
    volatile float centred = static_cast<float>(s) - c.mean;
    volatile float xhat = centred * c.inv;
    volatile float scaled = c.gamma * xhat;
    volatile float y = scaled + c.beta;
    return y >= 0.0f;
}

}  // namespace

extern "C" int bnn_bn_fold(const float* gamma, const float* beta, const float* mean, const float* var,
                           float eps, int64_t N, int64_t K, int32_t* thr, uint32_t* flip_bits) {
    const int64_t kMaxK = (int64_t(1) << 31) - 2;
    if (N < 0 || K < 0 || K > kMaxK) return BNN_ERR_INVALID_ARG;
    if (N == 0) return BNN_OK;
    if (!gamma || !beta || !mean || !var || !thr || !flip_bits) return BNN_ERR_INVALID_ARG;
    if (!std::isfinite(eps)) return BNN_ERR_INVALID_ARG;
    for (int64_t n = 0; n < N; ++n) {
        volatile float d = var[n] + eps;
        if (!std::isfinite(gamma[n]) || !std::isfinite(beta[n]) || !std::isfinite(mean[n]) ||
            !std::isfinite(var[n]) || !(d > 0.0f))
            return BNN_ERR_INVALID_ARG;
    }

    const int64_t words = (N + 31) / 32;
    for (int64_t w = 0; w < words; ++w) flip_bits[w] = 0u;

    for (int64_t n = 0; n < N; ++n) {
        Channel c;
        c.gamma = gamma[n];
        c.beta = beta[n];
        c.mean = mean[n];
        volatile float denom = std::sqrt(var[n] + eps);
        volatile float inv = 1.0f / denom;
        c.inv = inv;

        const bool at_lo = bn_nonneg(c, -K);
        const bool at_hi = bn_nonneg(c, K);
        int64_t t;          // bit(s) = (s >= t) XOR flip
        bool flip = false;
        if (at_lo == at_hi) {
            // Monotone and equal at both ends: constant over [-K, K].
            t = at_lo ? -K : K + 1;
        } else {
            // Bisection keeps pred(lo) == at_lo and pred(hi) == at_hi, lo < hi.
            int64_t lo = -K, hi = K;
            while (hi - lo > 1) {
                const int64_t mid = lo + (hi - lo) / 2;
                if (bn_nonneg(c, mid) == at_lo) lo = mid; else hi = mid;
            }
            t = hi;                     // first s whose bit differs from the bit at -K
            flip = at_lo;               // down-set: true below t, false from t on
        }
        thr[n] = static_cast<int32_t>(t);
        if (flip) flip_bits[n >> 5] |= 1u << (n & 31);
    }
    return BNN_OK;
}
