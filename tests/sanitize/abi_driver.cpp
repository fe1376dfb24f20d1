// Host-side checks of the C ABI's argument validation under AddressSanitizer and
// UndefinedBehaviorSanitizer.  This file is compiled together with csrc/api.cpp
// (host code sanitized); the kernel families are replaced by the stubs below, so
// nothing here needs a GPU.  It walks the rejection table of include/miconv.h,
// shape arithmetic near the integer limits and the error-text buffer.
#include <climits>
#include <cstdio>
#include <cstring>

#include "../../include/miconv.h"
#include "../../paper_1912_01703_amd/csrc/common.h"

namespace miconv {
static int g_launches = 0;
hipError_t direct_fwd(const Problem&, const void*, const void*, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t direct_bwd_data(const Problem&, const void*, const void*, float*, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t direct_bwd_weight(const Problem&, const void*, const void*, float*, hipStream_t) { ++g_launches; return hipSuccess; }
bool mfma_supports(int, const Problem& pr) { return pr.R == 3 && pr.groups == 1; }
size_t mfma_workspace_bytes(int pass, const Problem& pr) { return pass == 2 ? (size_t)pr.K * pr.Cg * pr.R * pr.S * 8 : 0; }
hipError_t mfma_run(int, const Problem&, const void*, const void*, float*, void*, hipStream_t, bool* fused) { ++g_launches; *fused = false; return hipSuccess; }
const char* mfma_path_name(int, const Problem&) { return "mfma/stub"; }
bool depthwise_supports(int, const Problem& pr) { return pr.groups == pr.C && pr.groups == pr.K && pr.groups > 1; }
size_t depthwise_workspace_bytes(int, const Problem&) { return 0; }
hipError_t depthwise_run(int, const Problem&, const void*, const void*, float*, void*, hipStream_t, bool* fused) { ++g_launches; *fused = true; return hipSuccess; }
const char* depthwise_path_name(int, const Problem&) { return "depthwise/stub"; }
static int g_epilogues = 0;
bool mfma_fuses_epilogue(int, const Problem&) { return false; }
bool depthwise_fuses_epilogue(int, const Problem&) { return true; }
hipError_t epilogue_run(int, const Problem&, void*, bool, hipStream_t) { ++g_epilogues; return hipSuccess; }
static int g_conversions = 0;
hipError_t convert_to_bf16(const float*, void*, size_t, hipStream_t) { ++g_conversions; return hipSuccess; }
bool mfma_writes_bf16(int, const Problem& pr, const void*, const void*) { return pr.C == 8; }
}  // namespace miconv

typedef int (*pass_fn)(const void*, const void*, void*, int, int, int, int, int, int, int, int, int, int, int, int, int, void*,
                       size_t, void*);

static int failures = 0;
#define EXPECT(cond)                                                                  \
    do {                                                                              \
        if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } \
    } while (0)

int main() {
    alignas(256) static char buf[4096];
    void* p = buf;
    const pass_fn fns[3] = {conv2d_fwd, conv2d_bwd_data, conv2d_bwd_weight};
    for (int f = 0; f < 3; ++f) {
        const pass_fn fn = fns[f];
        EXPECT(fn(p, p, p, 0, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 0, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 3, 3, 0, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, -1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 4, 2, 8, 4, 3, 3, 1, 1, 0, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(std::strstr(miconv_last_error(), "larger") != nullptr);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 3, 0, nullptr, 0, nullptr) == MICONV_ERR_GROUPS);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 0, 0, nullptr, 0, nullptr) == MICONV_ERR_GROUPS);
        EXPECT(fn(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 7, nullptr, 0, nullptr) == MICONV_ERR_DTYPE);
        // arithmetic at the integer limits: products are formed in 64 bits, nothing may overflow
        EXPECT(fn(p, p, p, INT_MAX, INT_MAX, INT_MAX, INT_MAX, INT_MAX, 1, 1, 1, 1, 0, 0, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 1, INT_MAX, INT_MAX, 1, 3, 3, 1, 1, INT_MAX, INT_MAX, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1, 1, 5, 5, 1, INT_MAX, INT_MAX, INT_MAX, INT_MAX, INT_MAX, INT_MAX, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(p, p, p, 1 << 20, 1 << 10, 64, 64, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_SHAPE);
        EXPECT(fn(nullptr, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_NULL);
        EXPECT(fn(p, nullptr, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_NULL);
        EXPECT(fn(p, p, nullptr, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_NULL);
    }
    EXPECT(miconv::g_launches == 0);
    // workspace rules (the stub family asks for 8 bytes per filter element in backward-weight)
    const size_t need = conv2d_workspace_bytes(2, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0);
    EXPECT(need == 4 * 4 * 9 * 8);
    EXPECT(conv2d_bwd_weight(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_WORKSPACE);
    EXPECT(conv2d_bwd_weight(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, p, need - 1, nullptr) == MICONV_ERR_WORKSPACE);
    EXPECT(conv2d_bwd_weight(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, buf + 64, need, nullptr) == MICONV_ERR_WORKSPACE);
    EXPECT(miconv::g_launches == 0);
    EXPECT(conv2d_bwd_weight(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, p, need, nullptr) == MICONV_OK);
    EXPECT(miconv::g_launches == 1 && miconv_last_algo(2) == MICONV_ALGO_MFMA);
    miconv::g_launches = 0;
    // bf16 results: a kernel that writes float needs room for its float result behind its own scratch memory
    EXPECT(conv2d_workspace_bytes(0, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT) == 1 * 4 * 8 * 8 * 4);
    EXPECT(conv2d_workspace_bytes(0, 1, 8, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT) == 0);    // (the stub writes bf16 itself)
    EXPECT(conv2d_workspace_bytes(2, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT) == need);  // dw stays float
    EXPECT(conv2d_fwd(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT, nullptr, 0, nullptr) == MICONV_ERR_WORKSPACE);
    EXPECT(conv2d_fwd(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT, p, 1024, nullptr) == MICONV_OK);
    EXPECT(miconv::g_conversions == 1);
    EXPECT(conv2d_fwd(p, p, p, 1, 8, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, MICONV_BF16_BF16OUT, nullptr, 0, nullptr) == MICONV_OK);
    EXPECT(miconv::g_conversions == 1);
    // dispatch and overrides
    EXPECT(std::strcmp(miconv_kernel_path(0, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0), "mfma/stub") == 0);
    EXPECT(std::strcmp(miconv_kernel_path(0, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 4, 0), "depthwise/stub") == 0);
    EXPECT(std::strcmp(miconv_kernel_path(0, 1, 4, 8, 8, 4, 5, 5, 1, 1, 2, 2, 1, 0), "direct") == 0);
    EXPECT(std::strcmp(miconv_kernel_path(7, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0), "none") == 0);
    EXPECT(miconv_set_algo(0, 99) == MICONV_ERR_DTYPE && miconv_set_algo(-1, 0) == MICONV_ERR_DTYPE);
    EXPECT(miconv_set_algo(0, MICONV_ALGO_DEPTHWISE) == MICONV_OK);
    EXPECT(conv2d_fwd(p, p, p, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0, nullptr, 0, nullptr) == MICONV_ERR_UNSUPPORTED);
    EXPECT(miconv_set_algo(0, MICONV_ALGO_AUTO) == MICONV_OK);
    EXPECT(conv2d_workspace_bytes(-3, 1, 4, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 0) == 0);
    // the error text is bounded: the longest message must still be terminated inside its buffer
    conv2d_fwd(p, p, p, INT_MIN, INT_MIN, INT_MIN, INT_MIN, INT_MIN, INT_MIN, INT_MIN, 1, 1, 0, 0, 1, 0, nullptr, 0, nullptr);
    EXPECT(std::strlen(miconv_last_error()) < 256);
    std::puts(failures ? "failed" : "ok");
    return failures ? 1 : 0;
}
