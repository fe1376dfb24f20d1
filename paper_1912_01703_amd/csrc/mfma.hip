// Dispatcher of the MFMA paths: which kernel family serves which pass.
#include "common.h"
namespace miconv {

bool mfma_supports(int pass, const Problem& pr) {
    if (pr.groups == pr.C && pr.groups == pr.K && pr.groups > 1) return false;  // depthwise: no contraction to speak of
    if (pass == 0 || pass == 1) return tile_supports(pass, pr);
    return false;
}

size_t mfma_workspace_bytes(int, const Problem&) { return 0; }

hipError_t mfma_run(int pass, const Problem& pr, const void* a, const void* b, float* out, void*, hipStream_t st) {
    if (pass == 0 || pass == 1) return tile_run(pass, pr, a, b, out, st);
    return hipErrorNotSupported;
}

}  // namespace miconv
