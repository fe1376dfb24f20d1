// Training-mode batch normalisation of NCHW fp32 tensors, forward and backward, for gfx950.
//
// With M = N*H*W and all sums over the elements of one channel c:
//   mean = sum x / M,  var = sum (x - mean)^2 / M,  inv_std = 1 / sqrt(var + eps),
//   y  = gamma (x - mean) inv_std + beta
//   dbeta = sum dy,  dgamma = sum dy (x - mean) inv_std,
//   dx = gamma inv_std (dy - dbeta / M - (x - mean) inv_std dgamma / M)
//
// The operator is bound by HBM bandwidth (a few flops per element), so the kernels are organised around how
// often a tensor crosses the memory interface:
//
// * Channel-resident kernels.  When a channel (N planes of H*W floats, C*H*W apart) fits into the registers of
//   one workgroup (up to 1024 threads x 8 units of 16 bytes = 32 768 floats), one workgroup per channel loads it
//   once, computes the statistics with the plain two-pass formulas out of its registers, and writes the result:
//   x (and dy) are read once, y (dx) written once - the algorithmic minimum.
// * Split kernels for larger channels: (1) workgroups of 256 threads take chunks of 2048 units of a channel and
//   leave partial statistics in the workspace (chunk mean, sum of squares about the chunk mean, count); (2) one
//   wave per channel merges the chunks in a fixed order in double precision (pairwise-merge formula for the sum
//   of squares, so nothing is lost to cancellation); (3) an element-wise kernel applies the result.  x is read
//   twice.
//
// A unit is four consecutive floats of a plane read with one 16-byte access when planes are multiples of four
// floats and the tensors 16-byte aligned, one float otherwise.  All reductions run in a fixed order (butterfly
// inside a wave, waves in order through LDS, chunks in order): results do not depend on launch timing.
#include "../../include/miconv.h"
#include "common.h"
#include <type_traits>

namespace miconv {
namespace {

struct BnArgs {
    const float* x;
    const float* dy;
    const float* gamma;
    const float* beta;
    const float* mean_in;      // backward: saved statistics
    const float* inv_std_in;
    float* y;                  // forward result / backward dx
    float* mean;
    float* inv_std;
    float* dgamma;
    float* dbeta;
    float* ws;
    int N, C, HW;
    int upp;                   // units per plane
    int U;                     // units per channel = N * upp
    int S;                     // chunks per channel (split kernels)
    int chunk;                 // units per chunk
    float eps, inv_M;
};

constexpr int kChunkUnits = 2048;      // split kernels: 256 threads x 8 units
constexpr int kResidentUnits = 8192;   // channel-resident kernels: at most 1024 threads x 8 units

template <int VEC>
__device__ __forceinline__ void load_unit(const float* p, float (&v)[VEC]) {
    if constexpr (VEC == 4) {
        const float4 t = *reinterpret_cast<const float4*>(p);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    } else {
        v[0] = *p;
    }
}
template <int VEC>
__device__ __forceinline__ void store_unit(float* p, const float (&v)[VEC]) {
    if constexpr (VEC == 4) *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    else *p = v[0];
}

// Element offset of unit u of channel c (u counts units through the channel's N planes).
template <int VEC>
__device__ __forceinline__ size_t unit_offset(const BnArgs& a, int c, int u) {
    const int n = u / a.upp, r = u - n * a.upp;
    return ((size_t)n * a.C + c) * a.HW + (size_t)r * VEC;
}

// Sum over the workgroup, the same value in every thread: butterfly inside each wave, then the waves in order.
template <int NW>
__device__ __forceinline__ float block_sum(float v, float* red) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    __syncthreads();   // red may still be read from the previous reduction
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = red[0];
#pragma unroll
    for (int w = 1; w < NW; ++w) s += red[w];
    return s;
}

// ---------------------------------------------------------------------------------- channel-resident kernels
template <int THREADS, int VPT, int VEC>
__global__ __launch_bounds__(THREADS) void bn_fwd_channel_kernel(BnArgs a) {
    __shared__ float red[THREADS / 64];
    const int c = blockIdx.x, tid = threadIdx.x;
    float v[VPT][VEC];
    size_t off[VPT];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int u = tid + i * THREADS;
        off[i] = u < a.U ? unit_offset<VEC>(a, c, u) : 0;
        if (u < a.U) {
            load_unit<VEC>(a.x + off[i], v[i]);
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k) v[i][k] = 0.f;
        }
    }
#pragma unroll
    for (int i = 0; i < VPT; ++i)
#pragma unroll
        for (int k = 0; k < VEC; ++k) sum += v[i][k];
    const float mean = block_sum<THREADS / 64>(sum, red) * a.inv_M;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i)
        if (tid + i * THREADS < a.U) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const float d = v[i][k] - mean;
                sq = fmaf(d, d, sq);
            }
        }
    const float var = block_sum<THREADS / 64>(sq, red) * a.inv_M;
    const float inv_std = 1.0f / sqrtf(var + a.eps);
    if (tid == 0) {
        a.mean[c] = mean;
        a.inv_std[c] = inv_std;
    }
    const float g = a.gamma[c] * inv_std, b = a.beta[c];
#pragma unroll
    for (int i = 0; i < VPT; ++i)
        if (tid + i * THREADS < a.U) {
            float o[VEC];
#pragma unroll
            for (int k = 0; k < VEC; ++k) o[k] = fmaf(v[i][k] - mean, g, b);
            store_unit<VEC>(a.y + off[i], o);
        }
}

template <int THREADS, int VPT, int VEC>
__global__ __launch_bounds__(THREADS) void bn_bwd_channel_kernel(BnArgs a) {
    __shared__ float red[THREADS / 64];
    const int c = blockIdx.x, tid = threadIdx.x;
    const float mean = a.mean_in[c], inv_std = a.inv_std_in[c];
    float xv[VPT][VEC], gv[VPT][VEC];
    size_t off[VPT];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int u = tid + i * THREADS;
        off[i] = u < a.U ? unit_offset<VEC>(a, c, u) : 0;
        if (u < a.U) {
            load_unit<VEC>(a.x + off[i], xv[i]);
            load_unit<VEC>(a.dy + off[i], gv[i]);
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k) { xv[i][k] = mean; gv[i][k] = 0.f; }
        }
    }
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i)
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            xv[i][k] = (xv[i][k] - mean) * inv_std;      // xhat from here on
            s1 += gv[i][k];
            s2 = fmaf(gv[i][k], xv[i][k], s2);
        }
    const float dbeta = block_sum<THREADS / 64>(s1, red);
    const float dgamma = block_sum<THREADS / 64>(s2, red);
    if (tid == 0) {
        a.dbeta[c] = dbeta;
        a.dgamma[c] = dgamma;
    }
    const float k1 = a.gamma[c] * inv_std, k2 = dbeta * a.inv_M, k3 = dgamma * a.inv_M;
#pragma unroll
    for (int i = 0; i < VPT; ++i)
        if (tid + i * THREADS < a.U) {
            float o[VEC];
#pragma unroll
            for (int k = 0; k < VEC; ++k) o[k] = k1 * ((gv[i][k] - k2) - xv[i][k] * k3);
            store_unit<VEC>(a.y + off[i], o);
        }
}

// ---------------------------------------------------------------------------------------------- split kernels
// (1) partial statistics of chunk s of channel c; workgroup id = c * S + s.
template <int VEC>
__global__ __launch_bounds__(256) void bn_fwd_partial_kernel(BnArgs a) {
    constexpr int VPT = kChunkUnits / 256;
    __shared__ float red[4];
    const int c = blockIdx.x / a.S, s = blockIdx.x - c * a.S, tid = threadIdx.x;
    const int u0 = s * a.chunk, u1 = min(a.U, u0 + a.chunk);
    float v[VPT][VEC];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int u = u0 + tid + i * 256;
        if (u < u1) {
            load_unit<VEC>(a.x + unit_offset<VEC>(a, c, u), v[i]);
        } else {
#pragma unroll
            for (int k = 0; k < VEC; ++k) v[i][k] = 0.f;
        }
#pragma unroll
        for (int k = 0; k < VEC; ++k) sum += v[i][k];
    }
    const float count = (float)((u1 - u0) * VEC);
    const float mean = block_sum<4>(sum, red) / count;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i)
        if (u0 + tid + i * 256 < u1) {
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                const float d = v[i][k] - mean;
                sq = fmaf(d, d, sq);
            }
        }
    const float m2 = block_sum<4>(sq, red);
    if (tid == 0) {
        float* o = a.ws + (size_t)blockIdx.x * 3;
        o[0] = mean; o[1] = m2; o[2] = count;
    }
}

// Sum over a wave in double precision, the same value in every lane.
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// (2) one wave per channel merges the chunks: mean = sum n_s mean_s / M, M2 = sum (M2_s + n_s (mean_s - mean)^2).
__global__ __launch_bounds__(256) void bn_fwd_finalize_kernel(BnArgs a) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= a.C) return;
    const float* p = a.ws + (size_t)c * a.S * 3;
    double wsum = 0.0;
    for (int s = lane; s < a.S; s += 64) wsum += (double)p[3 * s + 2] * (double)p[3 * s];
    const double M = (double)a.N * (double)a.HW;
    const double mean = wave_sum(wsum) / M;
    double m2 = 0.0;
    for (int s = lane; s < a.S; s += 64) {
        const double d = (double)p[3 * s] - mean;
        m2 += (double)p[3 * s + 1] + (double)p[3 * s + 2] * d * d;
    }
    const double var = wave_sum(m2) / M;
    if (lane == 0) {
        a.mean[c] = (float)mean;
        a.inv_std[c] = (float)(1.0 / sqrt(var + (double)a.eps));
    }
}

// (3) y = (x - mean) * (gamma inv_std) + beta; one workgroup per (image, channel) plane.
template <int VEC>
__global__ __launch_bounds__(256) void bn_fwd_apply_kernel(BnArgs a) {
    const int plane = blockIdx.x, c = plane % a.C;
    const float mean = a.mean[c], g = a.gamma[c] * a.inv_std[c], b = a.beta[c];
    const float* x = a.x + (size_t)plane * a.HW;
    float* y = a.y + (size_t)plane * a.HW;
    for (int r = threadIdx.x; r < a.upp; r += 256) {
        float v[VEC], o[VEC];
        load_unit<VEC>(x + (size_t)r * VEC, v);
#pragma unroll
        for (int k = 0; k < VEC; ++k) o[k] = fmaf(v[k] - mean, g, b);
        store_unit<VEC>(y + (size_t)r * VEC, o);
    }
}

// backward (1): partial sums of dy and dy * xhat over chunk s of channel c.
template <int VEC>
__global__ __launch_bounds__(256) void bn_bwd_partial_kernel(BnArgs a) {
    constexpr int VPT = kChunkUnits / 256;
    __shared__ float red[4];
    const int c = blockIdx.x / a.S, s = blockIdx.x - c * a.S, tid = threadIdx.x;
    const int u0 = s * a.chunk, u1 = min(a.U, u0 + a.chunk);
    const float mean = a.mean_in[c], inv_std = a.inv_std_in[c];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
        const int u = u0 + tid + i * 256;
        if (u < u1) {
            float xv[VEC], gv[VEC];
            const size_t off = unit_offset<VEC>(a, c, u);
            load_unit<VEC>(a.x + off, xv);
            load_unit<VEC>(a.dy + off, gv);
#pragma unroll
            for (int k = 0; k < VEC; ++k) {
                s1 += gv[k];
                s2 = fmaf(gv[k], (xv[k] - mean) * inv_std, s2);
            }
        }
    }
    const float t1 = block_sum<4>(s1, red);
    const float t2 = block_sum<4>(s2, red);
    if (tid == 0) {
        float* o = a.ws + (size_t)blockIdx.x * 2;
        o[0] = t1; o[1] = t2;
    }
}

// backward (2): one wave per channel adds the chunks' sums in double precision.
__global__ __launch_bounds__(256) void bn_bwd_finalize_kernel(BnArgs a) {
    const int c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (c >= a.C) return;
    const float* p = a.ws + (size_t)c * a.S * 2;
    double t1 = 0.0, t2 = 0.0;
    for (int s = lane; s < a.S; s += 64) {
        t1 += (double)p[2 * s];
        t2 += (double)p[2 * s + 1];
    }
    t1 = wave_sum(t1);
    t2 = wave_sum(t2);
    if (lane == 0) {
        a.dbeta[c] = (float)t1;
        a.dgamma[c] = (float)t2;
    }
}

// backward (3): dx = gamma inv_std (dy - dbeta / M - xhat dgamma / M); one workgroup per plane.
template <int VEC>
__global__ __launch_bounds__(256) void bn_bwd_apply_kernel(BnArgs a) {
    const int plane = blockIdx.x, c = plane % a.C;
    const float mean = a.mean_in[c], inv_std = a.inv_std_in[c];
    const float k1 = a.gamma[c] * inv_std, k2 = a.dbeta[c] * a.inv_M, k3 = a.dgamma[c] * a.inv_M;
    const float* x = a.x + (size_t)plane * a.HW;
    const float* dy = a.dy + (size_t)plane * a.HW;
    float* dx = a.y + (size_t)plane * a.HW;
    for (int r = threadIdx.x; r < a.upp; r += 256) {
        float xv[VEC], gv[VEC], o[VEC];
        load_unit<VEC>(x + (size_t)r * VEC, xv);
        load_unit<VEC>(dy + (size_t)r * VEC, gv);
#pragma unroll
        for (int k = 0; k < VEC; ++k) o[k] = k1 * ((gv[k] - k2) - ((xv[k] - mean) * inv_std) * k3);
        store_unit<VEC>(dx + (size_t)r * VEC, o);
    }
}

// ------------------------------------------------------------------------------------------------------ host
int bn_fail(int code, const char* msg) { return record_error(code, "%s", msg); }

int bn_validate(int N, int C, int H, int W, int dtype) {
    if (N < 1 || C < 1 || H < 1 || W < 1) return bn_fail(MICONV_ERR_SHAPE, "batchnorm2d: N, C, H, W must all be >= 1");
    if (dtype != MICONV_F32) return bn_fail(MICONV_ERR_DTYPE, "batchnorm2d: only MICONV_F32 tensors are supported");
    constexpr long long lim = 1ll << 31;
    long long count = 1;   // every factor is below 2^31 and the running product is clamped: nothing exceeds 2^62
    for (long long f : {(long long)N, (long long)C, (long long)H, (long long)W}) count = count >= lim ? lim : count * f;
    if (count >= lim) return bn_fail(MICONV_ERR_SHAPE, "batchnorm2d: tensor too large (limit 2^31 elements)");
    return MICONV_OK;
}

// Chunks per channel of the split kernels for a unit of `vec` floats; 0 when the channel-resident kernels run.
int bn_splits(int N, int HW, int vec) {
    const long long U = (long long)N * (HW / vec);
    if (U <= kResidentUnits) return 0;
    return (int)((U + kChunkUnits - 1) / kChunkUnits);
}

template <int VEC, bool BWD>
hipError_t launch_resident(const BnArgs& a, hipStream_t st) {
    // the smallest workgroup whose registers hold the channel
    auto go = [&](auto threads, auto vpt) {
        constexpr int T = decltype(threads)::value, V = decltype(vpt)::value;
        if constexpr (BWD) bn_bwd_channel_kernel<T, V, VEC><<<a.C, T, 0, st>>>(a);
        else bn_fwd_channel_kernel<T, V, VEC><<<a.C, T, 0, st>>>(a);
    };
    using std::integral_constant;
    if (a.U <= 256 * 2) go(integral_constant<int, 256>{}, integral_constant<int, 2>{});
    else if (a.U <= 256 * 4) go(integral_constant<int, 256>{}, integral_constant<int, 4>{});
    else if (a.U <= 512 * 4) go(integral_constant<int, 512>{}, integral_constant<int, 4>{});
    else if (a.U <= 512 * 8) go(integral_constant<int, 512>{}, integral_constant<int, 8>{});
    else go(integral_constant<int, 1024>{}, integral_constant<int, 8>{});
    return hipGetLastError();
}

template <int VEC>
hipError_t run_fwd(BnArgs a, hipStream_t st) {
    a.upp = a.HW / VEC;
    a.U = a.N * a.upp;
    a.S = bn_splits(a.N, a.HW, VEC);
    a.chunk = kChunkUnits;
    if (a.S == 0) return launch_resident<VEC, false>(a, st);
    bn_fwd_partial_kernel<VEC><<<a.C * a.S, 256, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bn_fwd_finalize_kernel<<<(a.C + 3) / 4, 256, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    bn_fwd_apply_kernel<VEC><<<a.N * a.C, 256, 0, st>>>(a);
    return hipGetLastError();
}

template <int VEC>
hipError_t run_bwd(BnArgs a, hipStream_t st) {
    a.upp = a.HW / VEC;
    a.U = a.N * a.upp;
    a.S = bn_splits(a.N, a.HW, VEC);
    a.chunk = kChunkUnits;
    if (a.S == 0) return launch_resident<VEC, true>(a, st);
    bn_bwd_partial_kernel<VEC><<<a.C * a.S, 256, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    bn_bwd_finalize_kernel<<<(a.C + 3) / 4, 256, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    bn_bwd_apply_kernel<VEC><<<a.N * a.C, 256, 0, st>>>(a);
    return hipGetLastError();
}

bool aligned16(const void* p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// vec = 1: what a call may need at most (the pointers, whose alignment picks the unit, are not known to the query);
// a call itself only insists on what the unit it picked needs.
size_t bn_workspace(int pass, int N, int C, int H, int W, int vec = 1) {
    const int s = bn_splits(N, H * W, vec);
    return (size_t)C * s * (pass == 0 ? 3 : 2) * sizeof(float);
}

int check_ws(size_t need, void* ws, size_t ws_bytes) {
    if (need == 0) return MICONV_OK;
    if (!ws) return bn_fail(MICONV_ERR_WORKSPACE, "batchnorm2d: workspace is NULL but required");
    if (ws_bytes < need) return bn_fail(MICONV_ERR_WORKSPACE, "batchnorm2d: workspace too small");
    if (reinterpret_cast<uintptr_t>(ws) % 256) return bn_fail(MICONV_ERR_WORKSPACE, "batchnorm2d: workspace must be 256-byte aligned");
    return MICONV_OK;
}

}  // namespace
}  // namespace miconv

extern "C" {

size_t batchnorm2d_workspace_bytes(int pass, int N, int C, int H, int W, int dtype) {
    if (pass < 0 || pass > 1 || miconv::bn_validate(N, C, H, W, dtype) != MICONV_OK) return 0;
    return miconv::bn_workspace(pass, N, C, H, W);
}

int batchnorm2d_fwd(const void* x, const float* gamma, const float* beta, void* y, float* save_mean, float* save_inv_std,
                    int N, int C, int H, int W, float eps, int dtype, void* workspace, size_t workspace_bytes,
                    void* hip_stream) {
    using namespace miconv;
    int rc = bn_validate(N, C, H, W, dtype);
    if (rc != MICONV_OK) return rc;
    if (!(eps >= 0.f)) return bn_fail(MICONV_ERR_SHAPE, "batchnorm2d_fwd: eps must be >= 0");
    if (!x || !gamma || !beta || !y || !save_mean || !save_inv_std) return bn_fail(MICONV_ERR_NULL, "batchnorm2d_fwd: NULL tensor");
    const bool vec = (H * W) % 4 == 0 && aligned16(x) && aligned16(y);
    if ((rc = check_ws(bn_workspace(0, N, C, H, W, vec ? 4 : 1), workspace, workspace_bytes)) != MICONV_OK) return rc;
    BnArgs a{};
    a.x = static_cast<const float*>(x); a.gamma = gamma; a.beta = beta;
    a.y = static_cast<float*>(y); a.mean = save_mean; a.inv_std = save_inv_std;
    a.ws = static_cast<float*>(workspace);
    a.N = N; a.C = C; a.HW = H * W; a.eps = eps;
    a.inv_M = (float)(1.0 / ((double)N * H * W));
    const hipError_t e = vec ? run_fwd<4>(a, static_cast<hipStream_t>(hip_stream)) : run_fwd<1>(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MICONV_OK : bn_fail(MICONV_ERR_LAUNCH, hipGetErrorString(e));
}

int batchnorm2d_bwd(const void* x, const void* dy, const float* gamma, const float* save_mean, const float* save_inv_std,
                    void* dx, float* dgamma, float* dbeta, int N, int C, int H, int W, int dtype, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    using namespace miconv;
    int rc = bn_validate(N, C, H, W, dtype);
    if (rc != MICONV_OK) return rc;
    if (!x || !dy || !gamma || !save_mean || !save_inv_std || !dx || !dgamma || !dbeta)
        return bn_fail(MICONV_ERR_NULL, "batchnorm2d_bwd: NULL tensor");
    const bool vec = (H * W) % 4 == 0 && aligned16(x) && aligned16(dy) && aligned16(dx);
    if ((rc = check_ws(bn_workspace(1, N, C, H, W, vec ? 4 : 1), workspace, workspace_bytes)) != MICONV_OK) return rc;
    BnArgs a{};
    a.x = static_cast<const float*>(x); a.dy = static_cast<const float*>(dy); a.gamma = gamma;
    a.mean_in = save_mean; a.inv_std_in = save_inv_std;
    a.y = static_cast<float*>(dx); a.dgamma = dgamma; a.dbeta = dbeta;
    a.ws = static_cast<float*>(workspace);
    a.N = N; a.C = C; a.HW = H * W;
    a.inv_M = (float)(1.0 / ((double)N * H * W));
    const hipError_t e = vec ? run_bwd<4>(a, static_cast<hipStream_t>(hip_stream)) : run_bwd<1>(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? MICONV_OK : bn_fail(MICONV_ERR_LAUNCH, hipGetErrorString(e));
}

}  // extern "C"
