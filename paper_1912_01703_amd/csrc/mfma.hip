// Placeholder dispatcher for the MFMA kernels (none registered yet).
#include "common.h"
namespace miconv {
bool mfma_supports(int, const Problem&) { return false; }
size_t mfma_workspace_bytes(int, const Problem&) { return 0; }
hipError_t mfma_run(int, const Problem&, const void*, const void*, float*, void*, hipStream_t) {
    return hipErrorNotSupported;
}
}  // namespace miconv
