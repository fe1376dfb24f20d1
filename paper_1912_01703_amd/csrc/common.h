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
    // Fused epilogues (null: none).  Forward: y = max(0, y + bias[k]).  Backward-data: dx = relu_mask > 0 ? dx : 0,
    // relu_mask shaped like x with the element type dtype names.
    const float* bias = nullptr;
    const void* relu_mask = nullptr;
    // The kernel is to write y / dx as bf16 (round to nearest even) instead of float: set only for kernel families
    // that say they can (mfma_writes_bf16); everything else writes float into scratch memory and is converted.
    bool out_bf16 = false;
};

// bf16 bit pattern -> float, exact.
__device__ __forceinline__ float bf16_to_float(uint16_t b) {
    return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
__device__ __forceinline__ float load_elem(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_elem(const uint16_t* p, size_t i) { return bf16_to_float(p[i]); }

// Records the text miconv_last_error() returns on this host thread and hands `code` back (api.cpp).
int record_error(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- device helpers shared by the kernel files ---------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v3u __attribute__((ext_vector_type(3)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// Raw buffer loads: the hardware compares the byte offset with the descriptor's size and returns 0 at or
// beyond it, so an element that must read as zero (outside the image or the tile, past the last channel,
// an absent filter) is given the offset kOob and costs neither a branch nor a select on the result.
// Every range a kernel describes this way is smaller than 2 GiB.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr unsigned kOob = 0x80000000u;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const float*) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0));
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const uint16_t*) {
    return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_raw_buffer_load_b16(r, byte_off, 0, 0)) << 16);
}

// ---- direct kernels (direct.hip): any valid problem -------------------------------------
hipError_t direct_fwd(const Problem& pr, const void* x, const void* w, float* y, hipStream_t st);
hipError_t direct_bwd_data(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st);
hipError_t direct_bwd_weight(const Problem& pr, const void* x, const void* dy, float* dw, hipStream_t st);


// ---- MFMA implicit-GEMM kernels (mfma_*.hip): dense and grouped layers ------------------
// pass: 0 forward, 1 backward-data, 2 backward-weight.  a/b are the two inputs
// of the pass in the order of the C ABI; out is y, dx or dw.
bool mfma_supports(int pass, const Problem& pr);
size_t mfma_workspace_bytes(int pass, const Problem& pr);
hipError_t mfma_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void* ws, hipStream_t st,
                    bool* fused_epilogue);
// The kernel family inside the MFMA paths that mfma_run would take ("none" if mfma_supports is false).
const char* mfma_path_name(int pass, const Problem& pr);

// Tiled forward / stride-1 backward-data kernels (mfma_tile.hip).
bool tile_supports(int pass, const Problem& pr);
hipError_t tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, hipStream_t st);

// bf16 matrix-core forward / stride-1 backward-data for 3x3 filters (mfma_bf16.hip); needs workspace.
bool bf16_tile_supports(int pass, const Problem& pr);
bool bf16_tile_accepts(int pass, const Problem& pr, const void* in0);   // ... and will not decline this source tensor
size_t bf16_tile_workspace_bytes(int pass, const Problem& pr);
hipError_t bf16_tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                         hipStream_t st);

// bf16 matrix-core 1x1 layers, all three passes (mfma_bf16_gemm.hip); needs workspace.
bool bf16_gemm_supports(int pass, const Problem& pr);
bool bf16_gemm_accepts(int pass, const Problem& pr, const void* in0, const void* in1);   // ... and will not decline these tensors
size_t bf16_gemm_workspace_bytes(int pass, const Problem& pr);
hipError_t bf16_gemm_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws, hipStream_t st);

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

// ---- epilogues (epilogue.hip) --------------------------------------------------------------
// Whether the kernel a pass is dispatched to applies the problem's epilogue in its own write-out; if not, the
// dispatcher runs epilogue_run over the finished output.
bool mfma_fuses_epilogue(int pass, const Problem& pr);
bool depthwise_fuses_epilogue(int pass, const Problem& pr);
hipError_t epilogue_run(int pass, const Problem& pr, void* out, bool out_is_bf16, hipStream_t st);
// float -> bf16 (round to nearest even), count elements.
hipError_t convert_to_bf16(const float* src, void* dst, size_t count, hipStream_t st);
// Whether the MFMA kernel this pass is dispatched to can write bf16 results itself, given the first input tensor.
bool mfma_writes_bf16(int pass, const Problem& pr, const void* in0, const void* in1);

// ---- depthwise kernels (depthwise.hip): groups == C == K, no MFMA ------------------------
bool depthwise_supports(int pass, const Problem& pr);
size_t depthwise_workspace_bytes(int pass, const Problem& pr);
// *fused_epilogue tells whether the launched kernel applied pr's epilogue itself.
hipError_t depthwise_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void* ws,
                         hipStream_t st, bool* fused_epilogue);
const char* depthwise_path_name(int pass, const Problem& pr);

}  // namespace miconv
