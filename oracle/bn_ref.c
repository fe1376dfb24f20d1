/*
 * CPU oracle for batch normalisation of NCHW tensors, forward and backward, in
 * training mode.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * benchmark's cpu_baseline leg may call this; the product path never does.
 * It shares no code, header, table or helper with the HIP library.
 *
 * The paper names the operator only once, as one of the operators in its
 * ResNet-50 execution trace (Section 6.1, Figure 1), next to convolution; it
 * does not define it.  What is computed here is the standard training-mode
 * definition.  With M = N*H*W and all sums over n, h, w of one channel c:
 *
 *   mean[c]    = (1/M) sum x
 *   var[c]     = (1/M) sum (x - mean[c])^2                 (biased)
 *   inv_std[c] = 1 / sqrt(var[c] + eps)
 *   xhat       = (x - mean[c]) * inv_std[c]
 *   y          = gamma[c] * xhat + beta[c]
 *
 * and the vector-Jacobian product of (x, gamma, beta) -> y, as the paper's
 * Section 4.2 requires of a backward function:
 *
 *   dbeta[c]   = sum dy
 *   dgamma[c]  = sum dy * xhat
 *   dx         = gamma[c] * inv_std[c] * (dy - dbeta[c]/M - xhat * dgamma[c]/M)
 *
 * Everything is fp64; x and dy may be fp32 (dtype 0), bf16 bit patterns
 * (dtype 1) or fp64 (dtype 2) and are widened exactly.  gamma and beta are
 * fp64.  The statistics are the plain two-pass formulas, one channel after
 * the other; the backward routine recomputes them from x.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

static inline double ldv(const void *base, size_t i, int dtype)
{
    if (dtype == 0) return (double)((const float *)base)[i];
    if (dtype == 1) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return ((const double *)base)[i];
}

static void channel_stats(const void *x, int N, int C, int HW, int c, int dtype, double eps,
                          double *mean, double *inv_std)
{
    const double M = (double)N * (double)HW;
    double sum = 0.0;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) sum += ldv(x, ((size_t)n * C + c) * HW + i, dtype);
    const double mu = sum / M;
    double sq = 0.0;
    for (int n = 0; n < N; ++n)
        for (int i = 0; i < HW; ++i) {
            const double d = ldv(x, ((size_t)n * C + c) * HW + i, dtype) - mu;
            sq += d * d;
        }
    *mean = mu;
    *inv_std = 1.0 / sqrt(sq / M + eps);
}

int batchnorm2d_fwd_ref(const void *x, const double *gamma, const double *beta,
                        double *y, double *mean, double *inv_std,
                        int N, int C, int H, int W, double eps, int dtype)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || !(eps >= 0.0)) return 1;
    const int HW = H * W;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        channel_stats(x, N, C, HW, c, dtype, eps, &mean[c], &inv_std[c]);
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t e = ((size_t)n * C + c) * HW + i;
                const double xhat = (ldv(x, e, dtype) - mean[c]) * inv_std[c];
                y[e] = gamma[c] * xhat + beta[c];
            }
    }
    return 0;
}

int batchnorm2d_bwd_ref(const void *x, const void *dy, const double *gamma,
                        double *dx, double *dgamma, double *dbeta,
                        int N, int C, int H, int W, double eps, int dtype)
{
    if (N < 1 || C < 1 || H < 1 || W < 1 || !(eps >= 0.0)) return 1;
    const int HW = H * W;
    const double M = (double)N * (double)HW;
#pragma omp parallel for schedule(static)
    for (int c = 0; c < C; ++c) {
        double mu, s;
        channel_stats(x, N, C, HW, c, dtype, eps, &mu, &s);
        double sum_dy = 0.0, sum_dy_xhat = 0.0;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t e = ((size_t)n * C + c) * HW + i;
                const double g = ldv(dy, e, dtype);
                sum_dy += g;
                sum_dy_xhat += g * ((ldv(x, e, dtype) - mu) * s);
            }
        dbeta[c] = sum_dy;
        dgamma[c] = sum_dy_xhat;
        for (int n = 0; n < N; ++n)
            for (int i = 0; i < HW; ++i) {
                const size_t e = ((size_t)n * C + c) * HW + i;
                const double xhat = (ldv(x, e, dtype) - mu) * s;
                dx[e] = gamma[c] * s * (ldv(dy, e, dtype) - sum_dy / M - xhat * sum_dy_xhat / M);
            }
    }
    return 0;
}
