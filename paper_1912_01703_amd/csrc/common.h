// Internal declarations shared by the host dispatcher and the kernel files.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace miconv {

// A validated convolution problem (see include/miconv.h for the operator).
struct Problem {
    int N, C, H, W, K, R, S;
    int sh, sw, ph, pw, groups;
    int P, Q, Cg, Kg;
    int dtype;  // 0 = fp32 inputs, 1 = bf16 inputs (fp32 accumulate and outputs)
};

// bf16 bit pattern -> float, exact.
__device__ __forceinline__ float bf16_to_float(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) { return bf16_to_float(p[i]); }

// ---- direct kernels (direct.hip): any valid problem -------------------------------------
hipError_t direct_fwd(const Problem& pr, const void* x, const void* w, float* y, hipStream_t st);
hipError_t direct_bwd_data(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st);
hipError_t direct_bwd_weight(const Problem& pr, const void* x, const void* dy, float* dw, hipStream_t st);


// ---- MFMA implicit-GEMM kernels (mfma_*.hip): dense and grouped layers ------------------
// pass: 0 forward, 1 backward-data, 2 backward-weight.  a/b are the two inputs
// of the pass in the order of the C ABI; out is y, dx or dw.
bool mfma_supports(int pass, const Problem& pr);
size_t mfma_workspace_bytes(int pass, const Problem& pr);
hipError_t mfma_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void* ws, hipStream_t st);

// Tiled forward / stride-1 backward-data kernels (mfma_tile.hip).
bool tile_supports(int pass, const Problem& pr);
hipError_t tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, hipStream_t st);

// bf16 matrix-core forward / stride-1 backward-data for 3x3 filters (mfma_bf16.hip); needs workspace.
bool bf16_tile_supports(int pass, const Problem& pr);
size_t bf16_tile_workspace_bytes(int pass, const Problem& pr);
hipError_t bf16_tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                         hipStream_t st);

// bf16 matrix-core backward-weight for 3x3 stride-1 filters (mfma_bf16_wgrad.hip); needs workspace.
bool bf16_wgrad_supports(const Problem& pr);
size_t bf16_wgrad_workspace_bytes(const Problem& pr);
hipError_t bf16_wgrad_run(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st);

// Strided backward-data on the tiled kernel, one launch per output phase (mfma_tile_phase.hip).
bool tile_phase_supports(const Problem& pr);
hipError_t tile_phase_run(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st);
// ... and, for 3x3 stride-2 padding-1 layers, in one launch whose four phases share the dy patch.
bool tile_merge2_supports(const Problem& pr);
hipError_t tile_merge2_run(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st);

// Few-input-channel, large strided filter layers (mfma_smallc.hip): forward and backward-weight.
bool smallc_supports(int pass, const Problem& pr);
size_t smallc_workspace_bytes(int pass, const Problem& pr);
hipError_t smallc_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                      hipStream_t st);

// Backward-weight kernels (mfma_wgrad.hip).  ws_bytes receives the partial-sum buffer size.
bool wgrad_supports(const Problem& pr, size_t* ws_bytes);
hipError_t wgrad_run(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st);

// ---- depthwise kernels (depthwise.hip): groups == C == K, no MFMA ------------------------
bool depthwise_supports(int pass, const Problem& pr);
size_t depthwise_workspace_bytes(int pass, const Problem& pr);
hipError_t depthwise_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void* ws,
                         hipStream_t st);

}  // namespace miconv
