/*
 * Runs the CPU oracle (oracle/conv_ref.c, compiled into this program with
 * -fsanitize=address,undefined) over small problems whose buffers are exactly
 * as large as the tensors, so that any read or write outside a tensor, any
 * signed overflow or misaligned access in the oracle aborts the program.
 * Prints one checksum per routine and problem; the test compares them with
 * the unsanitized library's results.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int conv2d_fwd_ref(const void *, const void *, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_bwd_data_ref(const void *, const void *, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_bwd_weight_ref(const void *, const void *, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_fwd_ref_at(const void *, const void *, const int64_t *, int64_t, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_bwd_data_ref_at(const void *, const void *, const int64_t *, int64_t, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_bwd_weight_ref_at(const void *, const void *, const int64_t *, int64_t, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_fwd_bias_relu_ref(const void *, const void *, const double *, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int conv2d_bwd_data_relu_ref(const void *, const void *, const void *, double *, int, int, int, int, int, int, int, int, int, int, int, int, int);
int batchnorm2d_fwd_ref(const void *, const double *, const double *, double *, double *, double *, int, int, int, int, double, int);
int batchnorm2d_bwd_ref(const void *, const void *, const double *, double *, double *, double *, int, int, int, int, double, int);

/* N C H W K R S sh sw ph pw groups */
static const int CASES[][12] = {
    {2, 3, 7, 6, 4, 3, 3, 1, 1, 1, 1, 1},
    {1, 4, 9, 8, 6, 3, 2, 2, 1, 0, 1, 2},
    {2, 6, 8, 11, 6, 1, 3, 1, 3, 0, 2, 3},
    {1, 2, 12, 12, 2, 5, 5, 2, 2, 2, 2, 2},
    {2, 3, 13, 9, 5, 4, 3, 3, 2, 1, 0, 1},
    {1, 8, 6, 6, 8, 3, 3, 1, 1, 1, 1, 8},
    {2, 5, 8, 8, 7, 3, 3, 3, 3, 0, 0, 1},
    {1, 2, 10, 7, 4, 3, 3, 1, 1, 3, 2, 1},
    {5, 1, 1, 1, 3, 1, 1, 1, 1, 0, 0, 1},
};

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s; }

/* element i of a test tensor: small integers, exactly representable in bf16, fp32 and fp64 */
static double val(uint32_t *s) { return (double)((int)(lcg(s) >> 24) % 17 - 8); }

static void *make(size_t n, int dtype, uint32_t seed)
{
    uint32_t s = seed;
    if (dtype == 0) {
        float *p = malloc(n * sizeof *p);
        for (size_t i = 0; i < n; ++i) p[i] = (float)val(&s);
        return p;
    }
    if (dtype == 1) {
        uint16_t *p = malloc(n * sizeof *p);
        for (size_t i = 0; i < n; ++i) {
            union { float f; uint32_t u; } c;
            c.f = (float)val(&s);
            p[i] = (uint16_t)(c.u >> 16);
        }
        return p;
    }
    double *p = malloc(n * sizeof *p);
    for (size_t i = 0; i < n; ++i) p[i] = val(&s);
    return p;
}

static double checksum(const double *v, size_t n)
{
    double c = 0.0;
    for (size_t i = 0; i < n; ++i) c += v[i] * (double)(i % 13 + 1);
    return c;
}

int main(void)
{
    const int ncases = (int)(sizeof CASES / sizeof CASES[0]);
    for (int ci = 0; ci < ncases; ++ci)
        for (int dtype = 0; dtype < 3; ++dtype) {
            const int *a = CASES[ci];
            const int N = a[0], C = a[1], H = a[2], W = a[3], K = a[4], R = a[5], S = a[6];
            const int sh = a[7], sw = a[8], ph = a[9], pw = a[10], g = a[11];
            const int P = (H + 2 * ph - R) / sh + 1, Q = (W + 2 * pw - S) / sw + 1;
            const size_t nx = (size_t)N * C * H * W, nw = (size_t)K * (C / g) * R * S, ny = (size_t)N * K * P * Q;
            void *x = make(nx, dtype, 11u + ci), *w = make(nw, dtype, 23u + ci), *dy = make(ny, dtype, 37u + ci);
            double *y = malloc(ny * sizeof *y), *dx = malloc(nx * sizeof *dx), *dw = malloc(nw * sizeof *dw);
            int rc = conv2d_fwd_ref(x, w, y, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            rc |= conv2d_bwd_data_ref(dy, w, dx, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            rc |= conv2d_bwd_weight_ref(x, dy, dw, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            if (rc) { fprintf(stderr, "oracle rejected case %d\n", ci); return 2; }
            /* every element again through the single-element variants */
            size_t nmax = nx > ny ? nx : ny;
            if (nw > nmax) nmax = nw;
            int64_t *idx = malloc(nmax * sizeof *idx);
            double *at = malloc(nmax * sizeof *at);
            for (size_t i = 0; i < nmax; ++i) idx[i] = (int64_t)i;
            int bad = 0;
            rc = conv2d_fwd_ref_at(x, w, idx, (int64_t)ny, at, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            for (size_t i = 0; i < ny; ++i) bad |= at[i] != y[i];
            rc |= conv2d_bwd_data_ref_at(dy, w, idx, (int64_t)nx, at, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            for (size_t i = 0; i < nx; ++i) bad |= at[i] != dx[i];
            rc |= conv2d_bwd_weight_ref_at(x, dy, idx, (int64_t)nw, at, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            for (size_t i = 0; i < nw; ++i) bad |= at[i] != dw[i];
            if (rc || bad) { fprintf(stderr, "single-element variants disagree on case %d\n", ci); return 3; }
            printf("%d %d %.17g %.17g %.17g\n", ci, dtype, checksum(y, ny), checksum(dx, nx), checksum(dw, nw));
            /* the fused epilogues and batch normalisation on the same tensors: consistency with the plain passes, and
             * the sanitizers watching every access */
            double *bias = malloc((size_t)K * sizeof *bias), *y2 = malloc(ny * sizeof *y2), *dx2 = malloc(nx * sizeof *dx2);
            for (int k = 0; k < K; ++k) bias[k] = (double)(k % 5) - 2.0;
            rc = conv2d_fwd_bias_relu_ref(x, w, bias, y2, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);
            for (size_t i = 0; i < ny; ++i) {
                const double v = y[i] + bias[(i / ((size_t)P * Q)) % K];
                bad |= y2[i] != (v > 0.0 ? v : 0.0);
            }
            rc |= conv2d_bwd_data_relu_ref(dy, w, x, dx2, N, C, H, W, K, R, S, sh, sw, ph, pw, g, dtype);   /* x as the activation */
            for (size_t i = 0; i < nx; ++i) bad |= dx2[i] != 0.0 && dx2[i] != dx[i];
            if (rc || bad) { fprintf(stderr, "fused epilogues disagree with the plain passes on case %d\n", ci); return 6; }
            double *gam = malloc((size_t)C * sizeof *gam), *bet = malloc((size_t)C * sizeof *bet), *mean = malloc((size_t)C * sizeof *mean),
                   *istd = malloc((size_t)C * sizeof *istd), *dgam = malloc((size_t)C * sizeof *dgam), *dbet = malloc((size_t)C * sizeof *dbet);
            for (int c = 0; c < C; ++c) { gam[c] = 1.0 + 0.25 * c; bet[c] = 0.5 - c; }
            void *gx = make(nx, dtype, 53u + ci);   /* an upstream gradient shaped like x */
            rc = batchnorm2d_fwd_ref(x, gam, bet, dx2, mean, istd, N, C, H, W, 1e-3, dtype);
            double worst = 0.0;
            for (int c = 0; c < C; ++c) {   /* with gamma = 1 + c/4, beta = 1/2 - c the channel mean of y is beta */
                double m = 0.0;
                for (int n = 0; n < N; ++n)
                    for (int i = 0; i < H * W; ++i) m += dx2[((size_t)n * C + c) * H * W + i];
                m = m / ((double)N * H * W) - bet[c];
                if (m < 0) m = -m;
                if (m > worst) worst = m;
            }
            rc |= batchnorm2d_bwd_ref(x, gx, gam, dx2, dgam, dbet, N, C, H, W, 1e-3, dtype);
            if (rc || worst > 1e-12) { fprintf(stderr, "batch normalisation failed on case %d (%g)\n", ci, worst); return 7; }
            free(bias); free(y2); free(dx2); free(gam); free(bet); free(mean); free(istd); free(dgam); free(dbet); free(gx);
            free(x); free(w); free(dy); free(y); free(dx); free(dw); free(idx); free(at);
        }
    /* rejected problems must be refused before any access */
    if (conv2d_fwd_ref(NULL, NULL, NULL, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 3, 0) != 1) return 4;
    if (conv2d_bwd_data_ref(NULL, NULL, NULL, 1, 4, 2, 2, 4, 5, 5, 1, 1, 0, 0, 1, 0) != 2) return 5;
    puts("ok");
    return 0;
}
