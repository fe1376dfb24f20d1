// Placeholder dispatcher for the depthwise kernels (none registered yet).
#include "common.h"
namespace miconv {
bool depthwise_supports(int, const Problem&) { return false; }
size_t depthwise_workspace_bytes(int, const Problem&) { return 0; }
hipError_t depthwise_run(int, const Problem&, const void*, const void*, float*, void*, hipStream_t) {
    return hipErrorNotSupported;
}
}  // namespace miconv
