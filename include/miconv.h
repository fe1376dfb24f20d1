/*
 * miconv -- 2D convolution (cross-correlation) for AMD MI355X (gfx950):
 * forward, backward-data and backward-weight behind a plain C ABI.
 *
 * The operator is the "2d convolution" the paper names among its built-in
 * functions (Section 4.1); the two backward entry points are the
 * vector-Jacobian products of the forward function with respect to its input
 * and its weight, which is what the paper requires of a backward function
 * (Section 4.2).  Arithmetic is 32-bit float as in the paper's benchmarks
 * (Section 6.3, Table 1), with a bf16-input / fp32-accumulate variant.
 *
 * Common conventions for the three compute entry points
 * ------------------------------------------------------
 *  Shapes     x [N][C][H][W], w [K][C/groups][R][S], y [N][K][P][Q] with
 *             P = floor((H + 2*pad_h - R)/stride_h) + 1 and Q likewise.
 *             dy is shaped like y, dx like x, dw like w.  Everything is
 *             contiguous row-major (NCHW / KCRS).  Output channel k belongs to
 *             group k / (K/groups) and reads input channels
 *             [g*C/groups, (g+1)*C/groups).  Dilation is 1; there is no bias.
 *  Padding    zeros, the same amount on both sides of an axis.
 *  dtype      MICONV_F32: x, w, dy are float.  MICONV_BF16_F32ACC: x, w, dy are
 *             bfloat16 bit patterns (uint16_t); products are accumulated in
 *             fp32.  Outputs (y, dx, dw) are float in both cases.
 *             MICONV_BF16_BF16OUT: as MICONV_BF16_F32ACC with y and dx stored
 *             as bfloat16 (dw remains float).  The 3x3 stride-1 kernels on the
 *             bf16 matrix cores write bfloat16 themselves; every other kernel
 *             writes float into the workspace (conv2d_workspace_bytes accounts
 *             for it, assuming x / dy and w start on 4-byte boundaries; a
 *             tensor that starts on an odd element makes those kernels step
 *             aside, and the call then needs room for a float result as
 *             well or returns MICONV_ERR_WORKSPACE) and a conversion pass
 *             follows.  Where a fused epilogue
 *             is applied by a separate pass to a result that is already
 *             bfloat16, the bias is added to the rounded value and the sum is
 *             rounded again.
 *  Pointers   x, w, dy, y, dx, dw and workspace are DEVICE pointers on the
 *             current HIP device.  The caller owns all of them; the library
 *             never allocates, frees or keeps them.  Inputs are read only.
 *             Outputs must not overlap inputs.  Every output element is
 *             overwritten (beta = 0), including dx positions no filter tap
 *             reaches (they become 0).
 *  workspace  scratch of at least conv2d_workspace_bytes(...) bytes for the
 *             same arguments, 256-byte aligned; may be NULL when that size
 *             is 0.  Its contents are undefined afterwards.  It holds the
 *             partial sums of a split backward-weight reduction and, for
 *             bfloat16 inputs on the bf16 matrix-core kernels, re-laid-out
 *             copies of the operands (up to the size of the inputs).
 *  stream     a hipStream_t passed as void* (NULL = the default stream).  All
 *             work is enqueued on it; the call returns without synchronising,
 *             so the host can run ahead of the device as in the paper's
 *             Section 5.2.
 *  Errors     the return value is a miconv_status.  On anything other than
 *             MICONV_OK nothing has been launched (arguments are validated
 *             first); miconv_last_error() then describes the problem.  No C++
 *             exception crosses this boundary.
 *  Limits     every tensor must have fewer than 2^31 elements.
 *  Threads    calls may be made from several host threads; the algorithm
 *             override, the last-algorithm record and the error text below
 *             are kept per host thread.
 */
#ifndef MICONV_H
#define MICONV_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Exported symbols: the library is built with hidden default visibility. */
#define MICONV_API __attribute__((visibility("default")))

typedef enum {
    MICONV_OK = 0,
    MICONV_ERR_NULL = 1,       /* a required pointer is NULL */
    MICONV_ERR_SHAPE = 2,      /* a dimension < 1, stride < 1, pad < 0, P or Q < 1, or a tensor >= 2^31 elements */
    MICONV_ERR_GROUPS = 3,     /* groups < 1, or C or K not divisible by groups */
    MICONV_ERR_DTYPE = 4,      /* unknown dtype / pass / algorithm code */
    MICONV_ERR_WORKSPACE = 5,  /* workspace NULL, misaligned or smaller than required */
    MICONV_ERR_LAUNCH = 6,     /* the HIP runtime refused a launch */
    MICONV_ERR_UNSUPPORTED = 7 /* a forced algorithm cannot run this problem */
} miconv_status;

typedef enum {
    MICONV_F32 = 0,          /* x, w, dy float; y, dx, dw float */
    MICONV_BF16_F32ACC = 1,  /* x, w, dy bfloat16, fp32 accumulation; y, dx, dw float */
    MICONV_BF16_BF16OUT = 2  /* as 1, but y and dx are written as bfloat16 (the fp32 sum rounded to nearest even);
                              * dw stays float.  act of conv2d_bwd_data_relu_mask is bfloat16 as for 1. */
} miconv_dtype;

typedef enum { MICONV_PASS_FWD = 0, MICONV_PASS_BWD_DATA = 1, MICONV_PASS_BWD_WEIGHT = 2 } miconv_pass;

typedef enum {
    MICONV_ALGO_AUTO = 0,      /* pick the fastest kernel that supports the problem */
    MICONV_ALGO_DIRECT = 1,    /* plain direct kernels: any valid problem, slow */
    MICONV_ALGO_MFMA = 2,      /* LDS-staged implicit GEMM on MFMA (dense / grouped layers) */
    MICONV_ALGO_DEPTHWISE = 3  /* bandwidth-bound stencil kernels, groups == C == K */
} miconv_algo;

/*
 * The "2d convolution" of the paper's Section 4.1 (the operator behind the
 * convolution layer of its Listing 1):
 * y[n,k,p,q] = sum_{c,r,s} x[n, g*Cg+c, p*stride_h-pad_h+r, q*stride_w-pad_w+s] * w[k,c,r,s]
 * (no filter flip; taps outside the image read zero).
 */
MICONV_API int conv2d_fwd(const void *x, const void *w, void *y,
               int N, int C, int H, int W, int K, int R, int S,
               int stride_h, int stride_w, int pad_h, int pad_w, int groups,
               int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward function of conv2d_fwd in the sense of the paper's Section 4.2: the
 * vector-Jacobian product of conv2d_fwd with respect to x,
 * dx[n,c,h,w] = sum over all (k,p,q,r,s) with p*stride_h-pad_h+r == h and
 * q*stride_w-pad_w+s == w of dy[n,k,p,q] * w[k,c,r,s].  N,C,H,W describe dx.
 */
MICONV_API int conv2d_bwd_data(const void *dy, const void *w, void *dx,
                    int N, int C, int H, int W, int K, int R, int S,
                    int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                    int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward function of conv2d_fwd in the sense of the paper's Section 4.2: the
 * vector-Jacobian product of conv2d_fwd with respect to w,
 * dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n, g*Cg+c, p*stride_h-pad_h+r, q*stride_w-pad_w+s].
 * The result does not depend on launch timing: partial sums are combined in a
 * fixed order (no floating-point atomics).
 */
MICONV_API int conv2d_bwd_weight(const void *x, const void *dy, void *dw,
                      int N, int C, int H, int W, int K, int R, int S,
                      int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                      int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * conv2d_fwd with the two operations the paper's model code puts around its
 * convolution layer (Section 4.1, first listing: the layer's per-channel bias
 * and the rectified linear unit applied to its output) folded into the
 * write-out:
 *   y[n,k,p,q] = max(0, conv2d_fwd(x, w)[n,k,p,q] + bias[k]).
 * bias: DEVICE pointer to K floats (float for both dtypes), read only.
 * Everything else as for conv2d_fwd.  Kernel families that have no epilogue
 * of their own run one more element-wise pass over y; miconv_epilogue_is_fused
 * tells which case applies.
 */
MICONV_API int conv2d_fwd_bias_relu(const void *x, const void *w, const float *bias, void *y,
                         int N, int C, int H, int W, int K, int R, int S,
                         int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                         int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * conv2d_bwd_data followed by the backward function (Section 4.2) of the
 * rectified linear unit that produced the convolution's input (Section 4.1):
 *   dx[n,c,h,w] = act[n,c,h,w] > 0 ? conv2d_bwd_data(dy, w)[n,c,h,w] : 0,
 * i.e. the vector-Jacobian product of z -> conv2d_fwd(max(0, z), w) with
 * respect to z, where act = max(0, z) is the tensor the forward pass was fed
 * (the derivative of max(0, .) at 0 is taken as 0).
 * act: DEVICE pointer, shaped like x ([N][C][H][W]) with the element type
 * dtype names, read only; it may be the forward pass's x itself.
 * Everything else as for conv2d_bwd_data.
 */
MICONV_API int conv2d_bwd_data_relu_mask(const void *dy, const void *w, const void *act, void *dx,
                              int N, int C, int H, int W, int K, int R, int S,
                              int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                              int dtype, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Host-only query: 1 when the kernel that conv2d_fwd_bias_relu (pass
 * MICONV_PASS_FWD) or conv2d_bwd_data_relu_mask (MICONV_PASS_BWD_DATA) runs
 * for these arguments applies the epilogue in its own write-out (given
 * 16-byte aligned tensors), 0 when a separate element-wise pass follows.
 */
MICONV_API int miconv_epilogue_is_fused(int pass,
                             int N, int C, int H, int W, int K, int R, int S,
                             int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                             int dtype);

/*
 * Batch normalisation of an NCHW tensor in training mode: the other operator
 * the paper names next to convolution in its ResNet-50 execution trace
 * (Section 6.1, Figure 1).  With M = N*H*W and sums over n, h, w of channel c:
 *   save_mean[c]    = sum x / M
 *   save_inv_std[c] = 1 / sqrt(sum (x - save_mean[c])^2 / M + eps)     (biased variance)
 *   y[n,c,h,w]      = gamma[c] * (x[n,c,h,w] - save_mean[c]) * save_inv_std[c] + beta[c]
 * x, y: DEVICE pointers to [N][C][H][W] floats; gamma, beta, save_mean,
 * save_inv_std: DEVICE pointers to C floats.  eps >= 0.  dtype must be
 * MICONV_F32.  workspace: at least batchnorm2d_workspace_bytes(0, ...) bytes,
 * 256-byte aligned (0 when a channel fits the registers of one workgroup:
 * N*H*W <= 32768 with 16-byte aligned tensors and H*W a multiple of 4).
 * Ownership, stream behaviour and error codes as for the convolution calls;
 * running statistics are not kept.  Results do not depend on launch timing.
 */
MICONV_API int batchnorm2d_fwd(const void *x, const float *gamma, const float *beta, void *y,
                    float *save_mean, float *save_inv_std,
                    int N, int C, int H, int W, float eps, int dtype,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Backward function of batchnorm2d_fwd in the sense of the paper's Section
 * 4.2: the vector-Jacobian product with respect to x, gamma and beta, given the
 * statistics batchnorm2d_fwd saved:
 *   dbeta[c]  = sum dy
 *   dgamma[c] = sum dy * xhat,        xhat = (x - save_mean[c]) * save_inv_std[c]
 *   dx        = gamma[c] * save_inv_std[c] * (dy - dbeta[c]/M - xhat * dgamma[c]/M)
 * x, dy, dx: [N][C][H][W] floats; gamma, save_mean, save_inv_std, dgamma,
 * dbeta: C floats; all DEVICE pointers.  workspace: at least
 * batchnorm2d_workspace_bytes(1, ...) bytes.
 */
MICONV_API int batchnorm2d_bwd(const void *x, const void *dy, const float *gamma,
                    const float *save_mean, const float *save_inv_std,
                    void *dx, float *dgamma, float *dbeta,
                    int N, int C, int H, int W, int dtype,
                    void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of workspace that batchnorm2d_fwd (pass 0) or batchnorm2d_bwd (pass 1) may need at most for these arguments
 * (tensors that are 16-byte aligned need less, and none at all when a channel fits one workgroup); 0 for invalid
 * arguments as well. */
MICONV_API size_t batchnorm2d_workspace_bytes(int pass, int N, int C, int H, int W, int dtype);

/*
 * conv2d_bwd_weight for callers that cannot allocate device memory (code under
 * HIP graph capture, serving loops, harnesses that forbid hipMalloc): the same
 * kernels and the same result, bit for bit, as conv2d_bwd_weight, but the scratch memory (the
 * partial sums of a split reduction) is a static device array inside the
 * library instead of a caller workspace.  The call allocates and frees
 * nothing.  Limits and rules:
 *  - the array holds 32 MiB per GPU (kept by every GPU the library runs on until
 *    the process ends); a problem whose conv2d_workspace_bytes(
 *    MICONV_PASS_BWD_WEIGHT, ...) exceeds that returns MICONV_ERR_WORKSPACE and
 *    launches nothing (all nine fp32 benchmark layers fit; bf16 layers that
 *    need re-laid-out operand copies do not);
 *  - all calls on one GPU share that GPU's array: calls that may overlap on one
 *    GPU (different streams or host threads) race and must be serialised by the caller;
 *  - the first call on each GPU looks up the array's device address
 *    (hipGetSymbolAddress); make that call outside graph capture.
 * Everything else (argument meaning, errors, stream behaviour) is as for
 * conv2d_bwd_weight.
 */
MICONV_API int conv2d_bwd_weight_static_ws(const void *x, const void *dy, void *dw,
                                int N, int C, int H, int W, int K, int R, int S,
                                int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                                int dtype, void *hip_stream);

/*
 * Bytes of workspace the given pass (a miconv_pass) needs for these arguments
 * under the current algorithm override.  Returns 0 for invalid arguments as
 * well; the compute call reports those.
 */
MICONV_API size_t conv2d_workspace_bytes(int pass,
                              int N, int C, int H, int W, int K, int R, int S,
                              int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                              int dtype);

/*
 * Host-only query: the kernel family the given pass would run for these
 * arguments under the calling thread's algorithm override, as a string with
 * static storage: "direct", "mfma/tile", "mfma/tile_phase", "mfma/tile_merge2",
 * "mfma/wgrad", "mfma/smallc", "mfma/bf16_tile", "mfma/bf16_wgrad",
 * "depthwise/strip", "depthwise/rows", "depthwise/lds"; "none" for invalid
 * arguments or a forced algorithm that cannot run the problem.  Whenever the
 * answer is not "none" the compute call has a kernel for the problem.
 */
MICONV_API const char *miconv_kernel_path(int pass,
                                          int N, int C, int H, int W, int K, int R, int S,
                                          int stride_h, int stride_w, int pad_h, int pad_w, int groups,
                                          int dtype);

/*
 * Measurement utility (used by the benchmark to state throughput against the
 * clock the GPU really ran at; the paper's Section 6 reports measured
 * throughput only).  Enqueues a one-wave kernel on hip_stream that runs for
 * about duration_us microseconds (1 .. 1 000 000) without touching memory and
 * then writes two uint64_t to `counts` (DEVICE pointer, 16 bytes, 8-byte
 * aligned): counts[0] = shader-clock cycles that passed, counts[1] = ticks of
 * the GPU's constant-rate counter that passed.  *wall_clock_khz (HOST pointer)
 * receives that counter's rate, so the average shader clock over the interval
 * is counts[0] / counts[1] * wall_clock_khz kHz.  Launch it on a stream other
 * than the one the measured kernels run on.  Returns a miconv_status.
 */
MICONV_API int miconv_sample_shader_clock(void *counts, unsigned duration_us, int *wall_clock_khz, void *hip_stream);

/*
 * Algorithm override for one pass (a miconv_algo), for the calling host thread
 * only (other threads keep their own setting; meant for tests and profiling).  With
 * MICONV_ALGO_AUTO (the default) every valid problem runs on some kernel.  A
 * forced algorithm that cannot run a problem makes the compute call return
 * MICONV_ERR_UNSUPPORTED.  Returns MICONV_OK or MICONV_ERR_DTYPE.
 */
MICONV_API int miconv_set_algo(int pass, int algo);

/* The miconv_algo the most recent successful call of that pass used on this
 * host thread (MICONV_ALGO_AUTO if none yet). */
MICONV_API int miconv_last_algo(int pass);

/* Description of the most recent failure on this host thread ("" if none).
 * The pointer stays valid until the thread's next failing call. */
MICONV_API const char *miconv_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MICONV_H */
