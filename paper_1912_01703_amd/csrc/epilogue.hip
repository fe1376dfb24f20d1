// Element-wise epilogues for the kernel families that do not apply them in their own write-out: one more pass
// over the finished output (16 bytes per lane where the tensor allows it).
//   forward:        y  = max(0, y + bias[k])
//   backward-data:  dx = act > 0 ? dx : 0
#include "common.h"

namespace miconv {
namespace {

__global__ __launch_bounds__(256) void bias_relu_kernel(float* __restrict__ y, const float* __restrict__ bias, int K, int plane,
                                                        size_t count) {
    // a thread owns four consecutive elements, which may straddle two planes
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 >= count) return;
    float v[4];
    const bool whole = i0 + 4 <= count && reinterpret_cast<uintptr_t>(y) % 16 == 0;
    if (whole) {
        const float4 t = *reinterpret_cast<const float4*>(y + i0);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        for (int j = 0; j < 4; ++j) v[j] = i0 + j < count ? y[i0 + j] : 0.f;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const size_t pl = (i0 + j) / (size_t)plane;
        v[j] = fmaxf(v[j] + bias[pl % (size_t)K], 0.f);
    }
    if (whole) {
        *reinterpret_cast<float4*>(y + i0) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
        for (int j = 0; j < 4; ++j)
            if (i0 + j < count) y[i0 + j] = v[j];
    }
}

template <typename T>
__global__ __launch_bounds__(256) void relu_mask_kernel(float* __restrict__ dx, const T* __restrict__ act, size_t count) {
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 >= count) return;
    if (i0 + 4 <= count && reinterpret_cast<uintptr_t>(dx) % 16 == 0 && reinterpret_cast<uintptr_t>(act) % (4 * sizeof(T)) == 0) {
        float4 t = *reinterpret_cast<const float4*>(dx + i0);
        float m[4];
        if constexpr (sizeof(T) == 4) {
            const float4 q = *reinterpret_cast<const float4*>(act + i0);
            m[0] = q.x; m[1] = q.y; m[2] = q.z; m[3] = q.w;
        } else {
            const uint2 q = *reinterpret_cast<const uint2*>(act + i0);
            m[0] = bf16_to_float(q.x & 0xFFFF); m[1] = bf16_to_float(q.x >> 16);
            m[2] = bf16_to_float(q.y & 0xFFFF); m[3] = bf16_to_float(q.y >> 16);
        }
        t.x = m[0] > 0.f ? t.x : 0.f; t.y = m[1] > 0.f ? t.y : 0.f;
        t.z = m[2] > 0.f ? t.z : 0.f; t.w = m[3] > 0.f ? t.w : 0.f;
        *reinterpret_cast<float4*>(dx + i0) = t;
    } else {
        for (size_t i = i0; i < count && i < i0 + 4; ++i) dx[i] = load_elem(act, i) > 0.f ? dx[i] : 0.f;
    }
}

// The same on results that are already bf16 (the bias is then added to the rounded value and the sum rounded again).
__device__ __forceinline__ uint16_t to_bf16(float f) {
    const unsigned u = __float_as_uint(f);
    return static_cast<uint16_t>((u + 0x7FFFu + ((u >> 16) & 1u)) >> 16);   // nearest, ties to even (finite values)
}

__global__ __launch_bounds__(256) void bias_relu_bf16_kernel(uint16_t* __restrict__ y, const float* __restrict__ bias, int K, int plane,
                                                             size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    y[i] = to_bf16(fmaxf(bf16_to_float(y[i]) + bias[(i / (size_t)plane) % (size_t)K], 0.f));
}

template <typename T>
__global__ __launch_bounds__(256) void relu_mask_bf16_kernel(uint16_t* __restrict__ dx, const T* __restrict__ act, size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    if (!(load_elem(act, i) > 0.f)) dx[i] = 0;
}

__global__ __launch_bounds__(256) void to_bf16_kernel(const float* __restrict__ src, uint16_t* __restrict__ dst, size_t count) {
    const size_t i0 = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i0 >= count) return;
    if (i0 + 4 <= count && reinterpret_cast<uintptr_t>(src) % 16 == 0 && reinterpret_cast<uintptr_t>(dst) % 8 == 0) {
        const float4 v = *reinterpret_cast<const float4*>(src + i0);
        uint2 o;
        o.x = (unsigned)to_bf16(v.x) | ((unsigned)to_bf16(v.y) << 16);
        o.y = (unsigned)to_bf16(v.z) | ((unsigned)to_bf16(v.w) << 16);
        *reinterpret_cast<uint2*>(dst + i0) = o;
    } else {
        for (size_t i = i0; i < count && i < i0 + 4; ++i) dst[i] = to_bf16(src[i]);
    }
}

}  // namespace

hipError_t convert_to_bf16(const float* src, void* dst, size_t count, hipStream_t st) {
    to_bf16_kernel<<<(unsigned)((count + 1023) / 1024), 256, 0, st>>>(src, static_cast<uint16_t*>(dst), count);
    return hipGetLastError();
}

hipError_t epilogue_run(int pass, const Problem& pr, void* outv, bool out_is_bf16, hipStream_t st) {
    if (out_is_bf16) {
        uint16_t* o16 = static_cast<uint16_t*>(outv);
        if (pass == 0 && pr.bias) {
            const size_t count = (size_t)pr.N * pr.K * pr.P * pr.Q;
            bias_relu_bf16_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(o16, pr.bias, pr.K, pr.P * pr.Q, count);
            return hipGetLastError();
        }
        if (pass == 1 && pr.relu_mask) {
            const size_t count = (size_t)pr.N * pr.C * pr.H * pr.W;
            const unsigned grid = (unsigned)((count + 255) / 256);
            if (pr.dtype == 0) relu_mask_bf16_kernel<float><<<grid, 256, 0, st>>>(o16, static_cast<const float*>(pr.relu_mask), count);
            else relu_mask_bf16_kernel<uint16_t><<<grid, 256, 0, st>>>(o16, static_cast<const uint16_t*>(pr.relu_mask), count);
            return hipGetLastError();
        }
        return hipSuccess;
    }
    float* out = static_cast<float*>(outv);
    if (pass == 0 && pr.bias) {
        const size_t count = (size_t)pr.N * pr.K * pr.P * pr.Q;
        bias_relu_kernel<<<(unsigned)((count + 1023) / 1024), 256, 0, st>>>(out, pr.bias, pr.K, pr.P * pr.Q, count);
        return hipGetLastError();
    }
    if (pass == 1 && pr.relu_mask) {
        const size_t count = (size_t)pr.N * pr.C * pr.H * pr.W;
        const unsigned grid = (unsigned)((count + 1023) / 1024);
        if (pr.dtype == 0) relu_mask_kernel<float><<<grid, 256, 0, st>>>(out, static_cast<const float*>(pr.relu_mask), count);
        else relu_mask_kernel<uint16_t><<<grid, 256, 0, st>>>(out, static_cast<const uint16_t*>(pr.relu_mask), count);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace miconv
