// Streamlining (Sec. 2.1 of the paper), host side: turn the floating-point operations that
// sit between an integer matrix product and the next activation quantizer into per-channel
// integer thresholds.  Runs once per layer when a network is prepared, in double precision
// on the CPU; nothing here touches the GPU.
//
//  * Sec. 2.1.2, "moving and collapsing linear transformations": the previous layer's
//    quantizer affine a_q T + b_q moves past the matrix product, W (a_q x + b_q) =
//    a_q (W x) + b_q rowsum(W), and joins alpha-scaling and batch normalisation in one
//    per-channel transform y = a[m] x + b[m] of the integer accumulator x.
//  * Sec. 2.1.3, "absorbing linear operations into thresholds": t_i <- (t_i - b) / a, and,
//    x being an integer, each threshold is rounded up.  The paper leaves a < 0 out; there the
//    inequality flips, a x + b >= t  <=>  -x >= (t - b) / |a|, so the channel is marked for
//    negation (the caller negates that weight row) and thresholds are computed for -x.
#include <cmath>
#include <cstdint>
#include <limits>

#include "bsgemm.h"

namespace {

int32_t clamp_to_i32(double v)
{
    if (std::isnan(v)) return std::numeric_limits<int32_t>::max();
    if (v >= 2147483647.0) return std::numeric_limits<int32_t>::max();
    if (v <= -2147483648.0) return std::numeric_limits<int32_t>::min();
    return static_cast<int32_t>(v);
}

}  // namespace

extern "C" bs_status bs_streamline_collapse(int64_t M, double a_q, double b_q, const int64_t *rowsum_w,
                                            const double *alpha, const double *gamma, const double *beta,
                                            const double *mu, const double *sigma, double *a, double *b)
{
    if (M <= 0 || !a || !b) return BS_ERR_INVALID_ARG;
    if ((gamma || beta || mu || sigma) && !(gamma && beta && mu && sigma)) return BS_ERR_INVALID_ARG;
    if (b_q != 0.0 && !rowsum_w) return BS_ERR_INVALID_ARG;
    for (int64_t m = 0; m < M; ++m) {
        const double al = alpha ? alpha[m] : 1.0;
        // z = alpha * (a_q * x + b_q * rowsum)
        double sa = al * a_q;
        double sb = al * b_q * (rowsum_w ? static_cast<double>(rowsum_w[m]) : 0.0);
        if (gamma) {  // y = gamma * (z - mu) / sigma + beta
            if (sigma[m] == 0.0) return BS_ERR_INVALID_ARG;
            const double g = gamma[m] / sigma[m];
            sa = g * sa;
            sb = g * (sb - mu[m]) + beta[m];
        }
        a[m] = sa;
        b[m] = sb;
    }
    return BS_OK;
}

extern "C" bs_status bs_streamline_thresholds(const double *t, int T, const double *a, const double *b, int64_t M,
                                              int32_t *thr, uint8_t *negate)
{
    if (!t || !a || !b || !thr || T <= 0 || M <= 0) return BS_ERR_INVALID_ARG;
    for (int64_t m = 0; m < M; ++m) {
        if (negate) negate[m] = 0;
        for (int i = 0; i < T; ++i) {
            int32_t v;
            if (a[m] > 0.0) {
                v = clamp_to_i32(std::ceil((t[i] - b[m]) / a[m]));
            } else if (a[m] < 0.0) {
                if (!negate) return BS_ERR_UNSUPPORTED;  // the caller must be able to negate the channel
                negate[m] = 1;
                v = clamp_to_i32(std::ceil((t[i] - b[m]) / -a[m]));
            } else {  // constant pre-activation: a threshold is either always or never reached
                v = (b[m] >= t[i]) ? std::numeric_limits<int32_t>::min() : std::numeric_limits<int32_t>::max();
            }
            thr[m * T + i] = v;
        }
    }
    return BS_OK;
}
