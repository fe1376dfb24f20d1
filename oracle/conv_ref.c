/*
 * CPU oracle for 2D cross-correlation (NCHW) and its two vector-Jacobian
 * products.  TEST INFRASTRUCTURE ONLY: tests, the smoke check and the
 * benchmark's cpu_baseline leg may call this; the product path never does.
 * It shares no code, header, table or helper with the HIP library.
 *
 * What is computed (the paper only names the operator -- "2d convolution",
 * Section 4.1 -- and says that a backward pass is the vector-Jacobian product
 * of its forward function, Section 4.2; arithmetic is 32-bit float, Table 1.
 * The operator definition itself -- cross-correlation, zero padding, floor
 * output size, contiguous channel groups -- is the standard one):
 *
 *   P = floor((H + 2*pad_h - R)/stride_h) + 1,  Q likewise,
 *   Cg = C/groups, Kg = K/groups, output channel k belongs to group k/Kg and
 *   sees input channels [g*Cg, (g+1)*Cg).
 *
 *   fwd        y [n,k,p,q] = sum_{c,r,s} x[n, g*Cg+c, p*sh-ph+r, q*sw-pw+s] * w[k,c,r,s]
 *   bwd_data   dx[n,c,h,w] = sum over every (k,p,q,r,s) whose tap lands on (h,w)
 *                            of dy[n,k,p,q] * w[k,c,r,s]          (VJP w.r.t. x)
 *   bwd_weight dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n, g*Cg+c, p*sh-ph+r, q*sw-pw+s]
 *                                                                 (VJP w.r.t. w)
 *
 * Layouts: x[N][C][H][W], w[K][Cg][R][S], y[N][K][P][Q]; dy as y, dx as x,
 * dw as w; all contiguous, row-major.  Taps that fall outside the image read
 * zero.  Inputs may be fp32 (dtype 0), bf16 bit patterns (dtype 1) or fp64
 * (dtype 2); every input is widened exactly to fp64, every product and sum is
 * fp64, and outputs are fp64.  No blocking, no reordering, no SIMD: each
 * routine is the definition written as seven nested loops.  OpenMP is used
 * only across independent outputs.
 *
 * The *_at variants evaluate the same definitions for a caller-supplied list
 * of flat output indices (used to spot-check layers too large to run whole).
 */
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

static inline double ld(const void *base, size_t i, int dtype)
{
    if (dtype == 0) {
        return (double)((const float *)base)[i];
    } else if (dtype == 1) {
        uint32_t bits = ((uint32_t)((const uint16_t *)base)[i]) << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return ((const double *)base)[i];
}

static inline int out_dim(int in, int pad, int filt, int stride)
{
    return (in + 2 * pad - filt) / stride + 1;
}

int convref_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ---------------------------------------------------------------- forward */
int conv2d_fwd_ref(const void *x, const void *w, double *y,
                   int N, int C, int H, int W, int K, int R, int S,
                   int stride_h, int stride_w, int pad_h, int pad_w,
                   int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            const int g = k / Kg;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    double acc = 0.0;
                    for (int c = 0; c < Cg; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int h = p * stride_h - pad_h + r;
                                const int v = q * stride_w - pad_w + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                const size_t xi = (((size_t)n * C + (size_t)g * Cg + c) * H + h) * W + v;
                                const size_t wi = (((size_t)k * Cg + c) * R + r) * S + s;
                                acc += ld(x, xi, dtype) * ld(w, wi, dtype);
                            }
                    y[(((size_t)n * K + k) * P + p) * Q + q] = acc;
                }
        }
    return 0;
}

/* ---------------------------------------------------- backward w.r.t. input
 * Written as a scatter over the forward loop nest: every forward product
 * x[..]*w[..] that feeds y[n,k,p,q] sends dy[n,k,p,q]*w[..] back to that x
 * position.  Images are independent, so only n is parallel. */
int conv2d_bwd_data_ref(const void *dy, const void *w, double *dx,
                        int N, int C, int H, int W, int K, int R, int S,
                        int stride_h, int stride_w, int pad_h, int pad_w,
                        int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;

#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *dxn = dx + (size_t)n * C * H * W;
        for (size_t i = 0; i < (size_t)C * H * W; ++i) dxn[i] = 0.0;
        for (int k = 0; k < K; ++k) {
            const int g = k / Kg;
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const double gy = ld(dy, (((size_t)n * K + k) * P + p) * Q + q, dtype);
                    for (int c = 0; c < Cg; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                const int h = p * stride_h - pad_h + r;
                                const int v = q * stride_w - pad_w + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                const size_t wi = (((size_t)k * Cg + c) * R + r) * S + s;
                                dxn[((size_t)(g * Cg + c) * H + h) * W + v] += gy * ld(w, wi, dtype);
                            }
                }
        }
    }
    return 0;
}

/* --------------------------------------------------- backward w.r.t. weight */
int conv2d_bwd_weight_ref(const void *x, const void *dy, double *dw,
                          int N, int C, int H, int W, int K, int R, int S,
                          int stride_h, int stride_w, int pad_h, int pad_w,
                          int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;

#pragma omp parallel for collapse(2) schedule(static)
    for (int k = 0; k < K; ++k)
        for (int c = 0; c < Cg; ++c) {
            const int g = k / Kg;
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    double acc = 0.0;
                    for (int n = 0; n < N; ++n)
                        for (int p = 0; p < P; ++p)
                            for (int q = 0; q < Q; ++q) {
                                const int h = p * stride_h - pad_h + r;
                                const int v = q * stride_w - pad_w + s;
                                if (h < 0 || h >= H || v < 0 || v >= W) continue;
                                const size_t xi = (((size_t)n * C + (size_t)g * Cg + c) * H + h) * W + v;
                                const size_t yi = (((size_t)n * K + k) * P + p) * Q + q;
                                acc += ld(dy, yi, dtype) * ld(x, xi, dtype);
                            }
                    dw[(((size_t)k * Cg + c) * R + r) * S + s] = acc;
                }
        }
    return 0;
}

/* ------------------------------------------------ single-element variants
 * idx[i] is a flat index into the corresponding full output tensor;
 * out[i] receives that element.  Each is the defining sum for one element. */
int conv2d_fwd_ref_at(const void *x, const void *w, const int64_t *idx, int64_t nidx, double *out,
                      int N, int C, int H, int W, int K, int R, int S,
                      int stride_h, int stride_w, int pad_h, int pad_w,
                      int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;
    (void)N;

#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        const int q = (int)(t % Q); t /= Q;
        const int p = (int)(t % P); t /= P;
        const int k = (int)(t % K); t /= K;
        const int n = (int)t;
        const int g = k / Kg;
        double acc = 0.0;
        for (int c = 0; c < Cg; ++c)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    const int h = p * stride_h - pad_h + r;
                    const int v = q * stride_w - pad_w + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    const size_t xi = (((size_t)n * C + (size_t)g * Cg + c) * H + h) * W + v;
                    const size_t wi = (((size_t)k * Cg + c) * R + r) * S + s;
                    acc += ld(x, xi, dtype) * ld(w, wi, dtype);
                }
        out[i] = acc;
    }
    return 0;
}

/* dx[n,c,h,v]: gather form.  Output (p,q) reaches (h,v) through tap (r,s)
 * exactly when h + pad_h - r = p*stride_h and v + pad_w - s = q*stride_w with
 * 0 <= p < P and 0 <= q < Q. */
int conv2d_bwd_data_ref_at(const void *dy, const void *w, const int64_t *idx, int64_t nidx, double *out,
                           int N, int C, int H, int W, int K, int R, int S,
                           int stride_h, int stride_w, int pad_h, int pad_w,
                           int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;
    (void)N;

#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        const int v = (int)(t % W); t /= W;
        const int h = (int)(t % H); t /= H;
        const int cc = (int)(t % C); t /= C;
        const int n = (int)t;
        const int g = cc / Cg, c = cc % Cg;
        double acc = 0.0;
        for (int kk = 0; kk < Kg; ++kk)
            for (int r = 0; r < R; ++r)
                for (int s = 0; s < S; ++s) {
                    const int hp = h + pad_h - r, vq = v + pad_w - s;
                    if (hp < 0 || vq < 0 || hp % stride_h || vq % stride_w) continue;
                    const int p = hp / stride_h, q = vq / stride_w;
                    if (p >= P || q >= Q) continue;
                    const int k = g * Kg + kk;
                    const size_t yi = (((size_t)n * K + k) * P + p) * Q + q;
                    const size_t wi = (((size_t)k * Cg + c) * R + r) * S + s;
                    acc += ld(dy, yi, dtype) * ld(w, wi, dtype);
                }
        out[i] = acc;
    }
    return 0;
}

int conv2d_bwd_weight_ref_at(const void *x, const void *dy, const int64_t *idx, int64_t nidx, double *out,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w,
                             int groups, int dtype)
{
    if (groups < 1 || C % groups || K % groups) return 1;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    if (P < 1 || Q < 1) return 2;
    const int Cg = C / groups, Kg = K / groups;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < nidx; ++i) {
        int64_t t = idx[i];
        const int s = (int)(t % S); t /= S;
        const int r = (int)(t % R); t /= R;
        const int c = (int)(t % Cg); t /= Cg;
        const int k = (int)t;
        const int g = k / Kg;
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int p = 0; p < P; ++p)
                for (int q = 0; q < Q; ++q) {
                    const int h = p * stride_h - pad_h + r;
                    const int v = q * stride_w - pad_w + s;
                    if (h < 0 || h >= H || v < 0 || v >= W) continue;
                    const size_t xi = (((size_t)n * C + (size_t)g * Cg + c) * H + h) * W + v;
                    const size_t yi = (((size_t)n * K + k) * P + p) * Q + q;
                    acc += ld(dy, yi, dtype) * ld(x, xi, dtype);
                }
        out[i] = acc;
    }
    return 0;
}

/* ------------------------------------------------------- fused epilogues
 * The paper's model code places a rectified linear unit directly behind its
 * convolution layer (Section 4.1, the forward function of its first listing),
 * and the layer it uses there carries a per-output-channel bias.  The two
 * routines below are the convolution passes above with that neighbour folded
 * in; each is the plain pass followed by the element-wise rule.
 *
 *   fwd_bias_relu   y[n,k,p,q]  = max(0, conv2d_fwd(x,w)[n,k,p,q] + bias[k])
 *   bwd_data_relu   dx[n,c,h,w] = conv2d_bwd_data(dy,w)[n,c,h,w]  if act[n,c,h,w] > 0, else 0
 *
 * The second one is the vector-Jacobian product, with respect to z, of
 * z -> conv2d_fwd(max(0,z), w) where act = max(0,z) is the activation the
 * convolution was fed (derivative of max(0,.) taken as 0 at 0).
 * bias is fp64 here; act has the element type `dtype` names and the shape of x.
 */
int conv2d_fwd_bias_relu_ref(const void *x, const void *w, const double *bias, double *y,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w,
                             int groups, int dtype)
{
    const int rc = conv2d_fwd_ref(x, w, y, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype);
    if (rc) return rc;
    const int P = out_dim(H, pad_h, R, stride_h);
    const int Q = out_dim(W, pad_w, S, stride_w);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < P * Q; ++i) {
                double *e = &y[((size_t)n * K + k) * P * Q + i];
                const double v = *e + bias[k];
                *e = v > 0.0 ? v : 0.0;
            }
    return 0;
}

int conv2d_bwd_data_relu_ref(const void *dy, const void *w, const void *act, double *dx,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w,
                             int groups, int dtype)
{
    const int rc = conv2d_bwd_data_ref(dy, w, dx, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype);
    if (rc) return rc;
    const size_t count = (size_t)N * C * H * W;
    for (size_t i = 0; i < count; ++i)
        if (!(ld(act, i, dtype) > 0.0)) dx[i] = 0.0;
    return 0;
}
