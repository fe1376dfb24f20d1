// Dispatcher of the MFMA paths: which kernel family serves which pass.
#include "common.h"
namespace miconv {

static bool is_depthwise(const Problem& pr) { return pr.groups == pr.C && pr.groups == pr.K && pr.groups > 1; }

bool mfma_supports(int pass, const Problem& pr) {
    if (is_depthwise(pr)) return false;  // one input channel per filter: nothing to contract
    if (smallc_supports(pass, pr)) return true;
    if (bf16_tile_supports(pass, pr)) return true;
    if (pass == 2 && bf16_wgrad_supports(pr)) return true;
    if (pass == 0) return tile_supports(pass, pr);
    if (pass == 1) return tile_supports(pass, pr) || tile_phase_supports(pr);
    size_t ws;
    return wgrad_supports(pr, &ws);
}

size_t mfma_workspace_bytes(int pass, const Problem& pr) {
    size_t ws = 0;
    if (is_depthwise(pr)) return 0;
    if (smallc_supports(pass, pr)) return smallc_workspace_bytes(pass, pr);
    if (bf16_tile_supports(pass, pr)) return bf16_tile_workspace_bytes(pass, pr);
    if (pass == 2 && bf16_wgrad_supports(pr)) return bf16_wgrad_workspace_bytes(pr);
    if (pass == 2) wgrad_supports(pr, &ws);
    return ws;
}

hipError_t mfma_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void* ws, hipStream_t st) {
    if (smallc_supports(pass, pr)) return smallc_run(pass, pr, a, b, out, ws, st);
    if (bf16_tile_supports(pass, pr)) return bf16_tile_run(pass, pr, a, b, out, ws, st);
    if (pass == 2 && bf16_wgrad_supports(pr)) return bf16_wgrad_run(pr, a, b, out, ws, st);
    if (pass == 0) return tile_run(pass, pr, a, b, out, st);
    if (pass == 1) {
        if (tile_supports(pass, pr)) return tile_run(pass, pr, a, b, out, st);
        return tile_merge2_supports(pr) ? tile_merge2_run(pr, a, b, out, st) : tile_phase_run(pr, a, b, out, st);
    }
    return wgrad_run(pr, a, b, out, ws, st);
}

}  // namespace miconv
