// Direct convolution kernels: one work-item per output element (forward,
// backward-data) or one workgroup per filter tap (backward-weight).  They accept
// every valid problem and serve as the fallback for shapes the tiled MFMA and
// depthwise kernels decline.  fp32 FMA accumulation; 64-bit addressing.
#include "common.h"

namespace miconv {
namespace {

constexpr int kThreads = 256;

template <typename T>
__global__ __launch_bounds__(kThreads) void direct_fwd_kernel(Problem pr, const T* __restrict__ x,
                                                              const T* __restrict__ w, float* __restrict__ y) {
    const size_t total = (size_t)pr.N * pr.K * pr.P * pr.Q;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        size_t t = i;
        const int q = (int)(t % pr.Q); t /= pr.Q;
        const int p = (int)(t % pr.P); t /= pr.P;
        const int k = (int)(t % pr.K); t /= pr.K;
        const int n = (int)t;
        const int g = k / pr.Kg;
        const int h0 = p * pr.sh - pr.ph, v0 = q * pr.sw - pr.pw;
        const T* xg = x + ((size_t)n * pr.C + (size_t)g * pr.Cg) * pr.H * pr.W;
        const T* wk = w + (size_t)k * pr.Cg * pr.R * pr.S;
        float acc = 0.f;
        for (int c = 0; c < pr.Cg; ++c) {
            for (int r = 0; r < pr.R; ++r) {
                const int h = h0 + r;
                if (h < 0 || h >= pr.H) continue;
                for (int s = 0; s < pr.S; ++s) {
                    const int v = v0 + s;
                    if (v < 0 || v >= pr.W) continue;
                    acc = fmaf(load_elem(xg, ((size_t)c * pr.H + h) * pr.W + v),
                               load_elem(wk, ((size_t)c * pr.R + r) * pr.S + s), acc);
                }
            }
        }
        y[i] = acc;
    }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void direct_bwd_data_kernel(Problem pr, const T* __restrict__ dy,
                                                                   const T* __restrict__ w,
                                                                   float* __restrict__ dx) {
    const size_t total = (size_t)pr.N * pr.C * pr.H * pr.W;
    const size_t step = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += step) {
        size_t t = i;
        const int v = (int)(t % pr.W); t /= pr.W;
        const int h = (int)(t % pr.H); t /= pr.H;
        const int cc = (int)(t % pr.C); t /= pr.C;
        const int n = (int)t;
        const int g = cc / pr.Cg, c = cc - g * pr.Cg;
        // Only taps r == (h + pad) mod stride (and likewise s) can reach this pixel.
        const int hr = h + pr.ph, vr = v + pr.pw;
        const int r_first = hr % pr.sh, s_first = vr % pr.sw;
        const T* dyg = dy + ((size_t)n * pr.K + (size_t)g * pr.Kg) * pr.P * pr.Q;
        const T* wg = w + (size_t)g * pr.Kg * pr.Cg * pr.R * pr.S;
        float acc = 0.f;
        for (int kk = 0; kk < pr.Kg; ++kk) {
            for (int r = r_first; r < pr.R; r += pr.sh) {
                const int p = (hr - r) / pr.sh;
                if (hr - r < 0 || p >= pr.P) continue;
                for (int s = s_first; s < pr.S; s += pr.sw) {
                    const int q = (vr - s) / pr.sw;
                    if (vr - s < 0 || q >= pr.Q) continue;
                    acc = fmaf(load_elem(dyg, ((size_t)kk * pr.P + p) * pr.Q + q),
                               load_elem(wg, (((size_t)kk * pr.Cg + c) * pr.R + r) * pr.S + s), acc);
                }
            }
        }
        dx[i] = acc;
    }
}

// One workgroup per dw element.  Waves walk (n,p) rows, lanes walk q; the
// per-lane sums are combined by a fixed shuffle tree and a fixed-order sum over
// waves, so the result is bit-reproducible.
template <typename T>
__global__ __launch_bounds__(kThreads) void direct_bwd_weight_kernel(Problem pr, const T* __restrict__ x,
                                                                     const T* __restrict__ dy,
                                                                     float* __restrict__ dw) {
    __shared__ float partial[kThreads / 64];
    const size_t total = (size_t)pr.K * pr.Cg * pr.R * pr.S;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (size_t e = blockIdx.x; e < total; e += gridDim.x) {
        size_t t = e;
        const int s = (int)(t % pr.S); t /= pr.S;
        const int r = (int)(t % pr.R); t /= pr.R;
        const int c = (int)(t % pr.Cg); t /= pr.Cg;
        const int k = (int)t;
        const int g = k / pr.Kg;
        float acc = 0.f;
        const int rows = pr.N * pr.P;
        for (int np = wave; np < rows; np += kThreads / 64) {
            const int n = np / pr.P, p = np - n * pr.P;
            const int h = p * pr.sh - pr.ph + r;
            if (h < 0 || h >= pr.H) continue;
            const T* xrow = x + (((size_t)n * pr.C + (size_t)g * pr.Cg + c) * pr.H + h) * pr.W;
            const T* dyrow = dy + (((size_t)n * pr.K + k) * pr.P + p) * pr.Q;
            for (int q = lane; q < pr.Q; q += 64) {
                const int v = q * pr.sw - pr.pw + s;
                if (v < 0 || v >= pr.W) continue;
                acc = fmaf(load_elem(dyrow, q), load_elem(xrow, v), acc);
            }
        }
        for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
        __syncthreads();  // previous iteration's readers are done with partial[]
        if (lane == 0) partial[wave] = acc;
        __syncthreads();
        if (threadIdx.x == 0) {
            float sum = 0.f;
            for (int i = 0; i < kThreads / 64; ++i) sum += partial[i];
            dw[e] = sum;
        }
    }
}

inline int grid_for(size_t total, int per_block, int cap) {
    size_t blocks = (total + per_block - 1) / per_block;
    if (blocks < 1) blocks = 1;
    if (blocks > (size_t)cap) blocks = cap;
    return (int)blocks;
}

}  // namespace

hipError_t direct_fwd(const Problem& pr, const void* x, const void* w, float* y, hipStream_t st) {
    const size_t total = (size_t)pr.N * pr.K * pr.P * pr.Q;
    const int grid = grid_for(total, kThreads, 1 << 20);
    if (pr.dtype == 0)
        direct_fwd_kernel<float><<<grid, kThreads, 0, st>>>(pr, (const float*)x, (const float*)w, y);
    else
        direct_fwd_kernel<uint16_t><<<grid, kThreads, 0, st>>>(pr, (const uint16_t*)x, (const uint16_t*)w, y);
    return hipGetLastError();
}

hipError_t direct_bwd_data(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st) {
    const size_t total = (size_t)pr.N * pr.C * pr.H * pr.W;
    const int grid = grid_for(total, kThreads, 1 << 20);
    if (pr.dtype == 0)
        direct_bwd_data_kernel<float><<<grid, kThreads, 0, st>>>(pr, (const float*)dy, (const float*)w, dx);
    else
        direct_bwd_data_kernel<uint16_t><<<grid, kThreads, 0, st>>>(pr, (const uint16_t*)dy, (const uint16_t*)w, dx);
    return hipGetLastError();
}

hipError_t direct_bwd_weight(const Problem& pr, const void* x, const void* dy, float* dw, hipStream_t st) {
    const size_t total = (size_t)pr.K * pr.Cg * pr.R * pr.S;
    const int grid = grid_for(total, 1, 1 << 20);
    if (pr.dtype == 0)
        direct_bwd_weight_kernel<float><<<grid, kThreads, 0, st>>>(pr, (const float*)x, (const float*)dy, dw);
    else
        direct_bwd_weight_kernel<uint16_t><<<grid, kThreads, 0, st>>>(pr, (const uint16_t*)x, (const uint16_t*)dy, dw);
    return hipGetLastError();
}

}  // namespace miconv
