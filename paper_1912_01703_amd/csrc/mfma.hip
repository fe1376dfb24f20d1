// Dispatcher of the MFMA paths: which kernel family serves which pass.
#include "common.h"
#include <cstring>
namespace miconv {

static bool is_depthwise(const Problem& pr) { return pr.groups == pr.C && pr.groups == pr.K && pr.groups > 1; }

// A 1x1 filter at stride 1 without padding does not couple pixels: the plane may be given any shape with the same
// number of pixels.  Planes whose width has no tuned instance are presented 56 pixels wide (112 x 112 = 224 x 56), which
// puts them on the full-row 16-byte paths of all three passes.
static Problem canonical(const Problem& in) {
    Problem pr = in;
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1 && pr.sw == 1 && pr.ph == 0 && pr.pw == 0 && pr.W != 14 && pr.W != 28 && pr.W != 56 &&
        pr.W > 7 && (pr.H * pr.W) % 56 == 0) {
        pr.H = pr.P = pr.H * pr.W / 56;
        pr.W = pr.Q = 56;
    }
    return pr;
}

bool mfma_supports(int pass, const Problem& in) {
    const Problem pr = canonical(in);
    if (is_depthwise(pr)) return false;  // one input channel per filter: nothing to contract
    if (bf16_gemm_supports(pass, in)) return true;
    if (smallc_supports(pass, pr)) return true;
    if (bf16_tile_supports(pass, pr)) return true;
    if (pass == 2 && bf16_wgrad_supports(pr)) return true;
    if (pass == 0) return tile_supports(pass, pr);
    if (pass == 1) return tile_supports(pass, pr) || tile_phase_supports(pr);
    size_t ws;
    return wgrad_supports(pr, &ws);
}

size_t mfma_workspace_bytes(int pass, const Problem& in) {
    const Problem pr = canonical(in);
    size_t ws = 0;
    if (is_depthwise(pr)) return 0;
    if (bf16_gemm_supports(pass, in)) {
        // (room for the fp32-matrix-core backward-weight kernel as well: it takes over when a tensor is only 2-byte aligned)
        if (pass == 2) wgrad_supports(pr, &ws);
        const size_t own = bf16_gemm_workspace_bytes(pass, in);
        return own > ws ? own : ws;
    }
    if (smallc_supports(pass, pr)) return smallc_workspace_bytes(pass, pr);
    if (bf16_tile_supports(pass, pr)) return bf16_tile_workspace_bytes(pass, pr);
    if (pass == 2 && bf16_wgrad_supports(pr)) {
        // (room for the fp32-matrix-core kernel as well: it takes over when a tensor is only 2-byte aligned)
        wgrad_supports(pr, &ws);
        const size_t own = bf16_wgrad_workspace_bytes(pr);
        return own > ws ? own : ws;
    }
    if (pass == 2) wgrad_supports(pr, &ws);
    return ws;
}

const char* mfma_path_name(int pass, const Problem& in) {
    const Problem pr = canonical(in);
    if (!mfma_supports(pass, in)) return "none";
    if (bf16_gemm_supports(pass, in)) return "mfma/bf16_gemm";
    if (smallc_supports(pass, pr)) return "mfma/smallc";
    if (bf16_tile_supports(pass, pr)) return "mfma/bf16_tile";
    if (pass == 2) return bf16_wgrad_supports(pr) ? "mfma/bf16_wgrad" : "mfma/wgrad";
    if (pass == 0 || tile_supports(pass, pr)) return "mfma/tile";
    return tile_merge2_supports(pr) ? "mfma/tile_merge2" : "mfma/tile_phase";
}

bool mfma_writes_bf16(int pass, const Problem& in, const void* in0, const void* in1) {
    if (pass < 2 && bf16_gemm_supports(pass, in)) return bf16_gemm_accepts(pass, in, in0, in1);
    const Problem pr = canonical(in);
    return pass < 2 && !smallc_supports(pass, pr) && bf16_tile_supports(pass, pr) && bf16_tile_accepts(pass, pr, in0);
}

// The kernels built on conv_tile_kernel and the bf16 1x1 product kernel apply bias + ReLU / the ReLU mask in their write-out.
bool mfma_fuses_epilogue(int pass, const Problem& in) {
    const char* path = mfma_path_name(pass, in);
    return std::strncmp(path, "mfma/tile", 9) == 0 || (pass < 2 && std::strcmp(path, "mfma/bf16_gemm") == 0);
}

hipError_t mfma_run(int pass, const Problem& in, const void* a, const void* b, float* out, void* ws, hipStream_t st,
                    bool* fused_epilogue) {
    const Problem pr = canonical(in);
    *fused_epilogue = mfma_fuses_epilogue(pass, in);
    if (bf16_gemm_supports(pass, in)) {
        // (declines tensors that are only 2-byte aligned: the kernels below take any alignment)
        const hipError_t e = bf16_gemm_run(pass, in, a, b, out, ws, st);
        if (e != hipErrorNotSupported) return e;
        *fused_epilogue = pass < 2;   // the fp32 tile kernels that take over apply the epilogue in their write-out
    }
    if (smallc_supports(pass, pr)) return smallc_run(pass, pr, a, b, out, ws, st);
    if (bf16_tile_supports(pass, pr)) {
        // (declines a source tensor that is only 2-byte aligned when it planned to read it in place: the kernels below
        // take any alignment)
        const hipError_t e = bf16_tile_run(pass, pr, a, b, out, ws, st);
        if (e != hipErrorNotSupported) return e;
        *fused_epilogue = true;   // the fp32 tile kernel that takes over applies the epilogue in its write-out
    }
    if (pass == 2 && bf16_wgrad_supports(pr)) {
        const hipError_t e = bf16_wgrad_run(pr, a, b, out, ws, st);
        if (e != hipErrorNotSupported) return e;
    }
    if (pass == 0) return tile_run(pass, pr, a, b, out, st);
    if (pass == 1) {
        if (tile_supports(pass, pr)) return tile_run(pass, pr, a, b, out, st);
        return tile_merge2_supports(pr) ? tile_merge2_run(pr, a, b, out, st) : tile_phase_run(pr, a, b, out, st);
    }
    return wgrad_run(pr, a, b, out, ws, st);
}

}  // namespace miconv
