// Host side of the C ABI declared in include/miconv.h: argument validation,
// algorithm selection, workspace sizing and launches on the caller's stream.
// Nothing here allocates device memory or synchronises.
#include "../../include/miconv.h"

#include <cstdarg>
#include <cstdio>
#include <mutex>

#include "common.h"

namespace {

using miconv::Problem;

thread_local char g_err[256] = "";
thread_local int g_last_algo[3] = {MICONV_ALGO_AUTO, MICONV_ALGO_AUTO, MICONV_ALGO_AUTO};
thread_local int g_forced[3] = {MICONV_ALGO_AUTO, MICONV_ALGO_AUTO, MICONV_ALGO_AUTO};

}  // namespace

namespace miconv {
int record_error(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace miconv

namespace {
using miconv::record_error;

// Scratch memory of conv2d_bwd_weight_static_ws: one array per GPU, held from the time the library's code is
// loaded on that GPU until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; the device address that call returns on the current device is what kernels are given.
constexpr size_t kStaticWsBytes = size_t(32) << 20;
__device__ __align__(256) unsigned char scratch[kStaticWsBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device); nullptr with the error recorded.
void* static_scratch() {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        record_error(MICONV_ERR_LAUNCH, "hipGetDevice failed or device index %d is out of range: %s", dev, hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            record_error(MICONV_ERR_LAUNCH, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Fills pr and returns MICONV_OK, or records why the arguments are invalid.
int make_problem(Problem& pr, int N, int C, int H, int W, int K, int R, int S, int sh, int sw, int ph, int pw,
                 int groups, int dtype) {
    if (N < 1 || C < 1 || H < 1 || W < 1 || K < 1 || R < 1 || S < 1)
        return record_error(MICONV_ERR_SHAPE, "N,C,H,W,K,R,S must all be >= 1 (got %d,%d,%d,%d,%d,%d,%d)", N, C, H, W, K, R, S);
    if (sh < 1 || sw < 1) return record_error(MICONV_ERR_SHAPE, "strides must be >= 1 (got %d,%d)", sh, sw);
    if (ph < 0 || pw < 0) return record_error(MICONV_ERR_SHAPE, "padding must be >= 0 (got %d,%d)", ph, pw);
    if (groups < 1 || C % groups || K % groups)
        return record_error(MICONV_ERR_GROUPS, "groups=%d must be >= 1 and divide C=%d and K=%d", groups, C, K);
    if (dtype != MICONV_F32 && dtype != MICONV_BF16_F32ACC && dtype != MICONV_BF16_BF16OUT)
        return record_error(MICONV_ERR_DTYPE, "unknown dtype %d", dtype);
    const long long hp = (long long)H + 2LL * ph - R, wq = (long long)W + 2LL * pw - S;
    if (hp < 0 || wq < 0)
        return record_error(MICONV_ERR_SHAPE, "filter %dx%d larger than padded input %dx%d (+2*%d,+2*%d)", R, S, H, W, ph, pw);
    const long long P = hp / sh + 1, Q = wq / sw + 1;
    constexpr long long lim = 1LL << 31;
    // products of four factors: each factor and the running product are clamped to 2^31, so nothing exceeds 2^62
    const auto count = [](long long a, long long b, long long c, long long d) {
        long long v = 1;
        for (long long f : {a, b, c, d}) v = v >= lim ? lim : v * (f >= lim ? lim : f);
        return v >= lim ? lim : v;
    };
    const long long nx = count(N, C, H, W), ny = count(N, K, P, Q), nw = count(K, C / groups, R, S);
    if (nx >= lim || ny >= lim || nw >= lim)
        return record_error(MICONV_ERR_SHAPE, "tensor too large: x=%lld y=%lld w=%lld elements (counts are capped at the limit, 2^31)", nx, ny, nw);
    pr.N = N; pr.C = C; pr.H = H; pr.W = W; pr.K = K; pr.R = R; pr.S = S;
    pr.sh = sh; pr.sw = sw; pr.ph = ph; pr.pw = pw; pr.groups = groups;
    pr.P = (int)P; pr.Q = (int)Q; pr.Cg = C / groups; pr.Kg = K / groups;
    pr.dtype = dtype == MICONV_F32 ? 0 : 1;   // element type of the inputs; the bf16-output variant is the caller's business
    return MICONV_OK;
}

// The algorithm that will run this pass, or -1 when the forced one cannot.
int choose_algo(int pass, const Problem& pr) {
    const int forced = g_forced[pass];
    const bool dw_ok = miconv::depthwise_supports(pass, pr);
    const bool mfma_ok = miconv::mfma_supports(pass, pr);
    switch (forced) {
        case MICONV_ALGO_DIRECT: return MICONV_ALGO_DIRECT;
        case MICONV_ALGO_MFMA: return mfma_ok ? MICONV_ALGO_MFMA : -1;
        case MICONV_ALGO_DEPTHWISE: return dw_ok ? MICONV_ALGO_DEPTHWISE : -1;
        default: break;
    }
    if (dw_ok) return MICONV_ALGO_DEPTHWISE;
    if (mfma_ok) return MICONV_ALGO_MFMA;
    return MICONV_ALGO_DIRECT;
}

size_t workspace_for(int pass, int algo, const Problem& pr) {
    if (algo == MICONV_ALGO_MFMA) return miconv::mfma_workspace_bytes(pass, pr);
    if (algo == MICONV_ALGO_DEPTHWISE) return miconv::depthwise_workspace_bytes(pass, pr);
    return 0;
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// bf16 results (y, dx) from a kernel that only writes float: the float result goes to scratch memory behind the kernel's
// own and is converted from there.
bool wants_bf16_out(int pass, int dtype) { return dtype == MICONV_BF16_BF16OUT && pass != MICONV_PASS_BWD_WEIGHT; }
size_t out_elems(int pass, const Problem& pr) {
    return pass == MICONV_PASS_FWD ? (size_t)pr.N * pr.K * pr.P * pr.Q : (size_t)pr.N * pr.C * pr.H * pr.W;
}
// in0 == nullptr: the query, which assumes a first input tensor that is at least 4-byte aligned
size_t total_workspace(int pass, int algo, const Problem& pr, int dtype, const void* in0, const void* in1, bool* native_bf16) {
    const size_t own = workspace_for(pass, algo, pr);
    *native_bf16 = false;
    if (!wants_bf16_out(pass, dtype)) return own;
    *native_bf16 = algo == MICONV_ALGO_MFMA && miconv::mfma_writes_bf16(pass, pr, in0, in1);
    return *native_bf16 ? own : round256(own) + out_elems(pass, pr) * sizeof(float);
}

int run(int pass, const void* a, const void* b, void* out, int N, int C, int H, int W, int K, int R, int S, int sh,
        int sw, int ph, int pw, int groups, int dtype, void* ws, size_t ws_bytes, void* stream,
        bool static_ws = false, bool with_epilogue = false, const void* epilogue_arg = nullptr) {
    static const char* const in_names[3][2] = {{"x", "w"}, {"dy", "w"}, {"x", "dy"}};
    static const char* const out_names[3] = {"y", "dx", "dw"};
    Problem pr;
    const int rc = make_problem(pr, N, C, H, W, K, R, S, sh, sw, ph, pw, groups, dtype);
    if (rc != MICONV_OK) return rc;
    if (!a) return record_error(MICONV_ERR_NULL, "%s is NULL", in_names[pass][0]);
    if (!b) return record_error(MICONV_ERR_NULL, "%s is NULL", in_names[pass][1]);
    if (!out) return record_error(MICONV_ERR_NULL, "%s is NULL", out_names[pass]);
    if (with_epilogue) {
        if (!epilogue_arg) return record_error(MICONV_ERR_NULL, "%s is NULL", pass == MICONV_PASS_FWD ? "bias" : "act");
        if (pass == MICONV_PASS_FWD) pr.bias = static_cast<const float*>(epilogue_arg);
        else pr.relu_mask = epilogue_arg;
    }
    const int algo = choose_algo(pass, pr);
    if (algo < 0)
        return record_error(MICONV_ERR_UNSUPPORTED, "forced algorithm %d cannot run this problem (pass %d)",
                    g_forced[pass], pass);
    bool native_bf16 = false;
    const bool bf16_out = wants_bf16_out(pass, dtype);
    const size_t need = total_workspace(pass, algo, pr, dtype, a, b, &native_bf16);
    if (static_ws) {
        if (need > kStaticWsBytes)
            return record_error(MICONV_ERR_WORKSPACE, "this problem needs %zu bytes of scratch memory, the static array holds %zu: "
                        "call conv2d_bwd_weight with a workspace instead", need, kStaticWsBytes);
        ws = need > 0 ? static_scratch() : nullptr;
        if (need > 0 && !ws) return MICONV_ERR_LAUNCH;
    } else if (need > 0) {
        if (!ws) return record_error(MICONV_ERR_WORKSPACE, "workspace is NULL but %zu bytes are required", need);
        if (ws_bytes < need) return record_error(MICONV_ERR_WORKSPACE, "workspace has %zu bytes, %zu required", ws_bytes, need);
        if (reinterpret_cast<uintptr_t>(ws) % 256)
            return record_error(MICONV_ERR_WORKSPACE, "workspace must be 256-byte aligned");
    }
    hipStream_t st = static_cast<hipStream_t>(stream);
    hipError_t e = hipSuccess;
    bool fused = false;
    // where the kernel writes: the caller's tensor, or (bf16 results from a float-only kernel) the staging area
    const bool staged = bf16_out && !native_bf16;
    float* o = staged ? reinterpret_cast<float*>(static_cast<unsigned char*>(ws) + round256(workspace_for(pass, algo, pr)))
                      : static_cast<float*>(out);
    pr.out_bf16 = native_bf16;
    if (algo == MICONV_ALGO_DIRECT) {
        if (pass == MICONV_PASS_FWD) e = miconv::direct_fwd(pr, a, b, o, st);
        else if (pass == MICONV_PASS_BWD_DATA) e = miconv::direct_bwd_data(pr, a, b, o, st);
        else e = miconv::direct_bwd_weight(pr, a, b, o, st);
    } else if (algo == MICONV_ALGO_MFMA) {
        e = miconv::mfma_run(pass, pr, a, b, o, ws, st, &fused);
    } else {
        e = miconv::depthwise_run(pass, pr, a, b, o, ws, st, &fused);
    }
    // kernels without an epilogue of their own: one element-wise pass over the finished output
    if (e == hipSuccess && with_epilogue && !fused) e = miconv::epilogue_run(pass, pr, o, native_bf16, st);
    if (e == hipSuccess && staged) e = miconv::convert_to_bf16(o, out, out_elems(pass, pr), st);
    if (e != hipSuccess) return record_error(MICONV_ERR_LAUNCH, "HIP launch failed: %s", hipGetErrorString(e));
    g_last_algo[pass] = algo;
    return MICONV_OK;
}

}  // namespace

extern "C" {

int conv2d_fwd(const void* x, const void* w, void* y, int N, int C, int H, int W, int K, int R, int S, int stride_h,
               int stride_w, int pad_h, int pad_w, int groups, int dtype, void* workspace, size_t workspace_bytes,
               void* hip_stream) {
    return run(MICONV_PASS_FWD, x, w, y, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype,
               workspace, workspace_bytes, hip_stream);
}

int conv2d_bwd_data(const void* dy, const void* w, void* dx, int N, int C, int H, int W, int K, int R, int S,
                    int stride_h, int stride_w, int pad_h, int pad_w, int groups, int dtype, void* workspace,
                    size_t workspace_bytes, void* hip_stream) {
    return run(MICONV_PASS_BWD_DATA, dy, w, dx, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype,
               workspace, workspace_bytes, hip_stream);
}

int conv2d_bwd_weight(const void* x, const void* dy, void* dw, int N, int C, int H, int W, int K, int R, int S,
                      int stride_h, int stride_w, int pad_h, int pad_w, int groups, int dtype, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
    return run(MICONV_PASS_BWD_WEIGHT, x, dy, dw, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
               dtype, workspace, workspace_bytes, hip_stream);
}

int conv2d_bwd_weight_static_ws(const void* x, const void* dy, void* dw, int N, int C, int H, int W, int K, int R, int S,
                                int stride_h, int stride_w, int pad_h, int pad_w, int groups, int dtype,
                                void* hip_stream) {
    return run(MICONV_PASS_BWD_WEIGHT, x, dy, dw, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups,
               dtype, nullptr, 0, hip_stream, true);
}

int conv2d_fwd_bias_relu(const void* x, const void* w, const float* bias, void* y, int N, int C, int H, int W, int K, int R,
                         int S, int stride_h, int stride_w, int pad_h, int pad_w, int groups, int dtype, void* workspace,
                         size_t workspace_bytes, void* hip_stream) {
    return run(MICONV_PASS_FWD, x, w, y, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype,
               workspace, workspace_bytes, hip_stream, false, true, bias);
}

int conv2d_bwd_data_relu_mask(const void* dy, const void* w, const void* act, void* dx, int N, int C, int H, int W, int K,
                              int R, int S, int stride_h, int stride_w, int pad_h, int pad_w, int groups, int dtype,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
    return run(MICONV_PASS_BWD_DATA, dy, w, dx, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype,
               workspace, workspace_bytes, hip_stream, false, true, act);
}

int miconv_epilogue_is_fused(int pass, int N, int C, int H, int W, int K, int R, int S, int stride_h, int stride_w, int pad_h,
                             int pad_w, int groups, int dtype) {
    if (pass != MICONV_PASS_FWD && pass != MICONV_PASS_BWD_DATA) return 0;
    Problem pr;
    if (make_problem(pr, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype) != MICONV_OK) return 0;
    switch (choose_algo(pass, pr)) {
        case MICONV_ALGO_MFMA: return miconv::mfma_fuses_epilogue(pass, pr) ? 1 : 0;
        case MICONV_ALGO_DEPTHWISE: return miconv::depthwise_fuses_epilogue(pass, pr) ? 1 : 0;
        default: return 0;
    }
}

size_t conv2d_workspace_bytes(int pass, int N, int C, int H, int W, int K, int R, int S, int stride_h, int stride_w,
                              int pad_h, int pad_w, int groups, int dtype) {
    if (pass < 0 || pass > 2) return 0;
    Problem pr;
    if (make_problem(pr, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype) != MICONV_OK) return 0;
    const int algo = choose_algo(pass, pr);
    if (algo < 0) return 0;
    bool native;
    return total_workspace(pass, algo, pr, dtype, nullptr, nullptr, &native);
}

const char* miconv_kernel_path(int pass, int N, int C, int H, int W, int K, int R, int S, int stride_h, int stride_w,
                               int pad_h, int pad_w, int groups, int dtype) {
    if (pass < 0 || pass > 2) return "none";
    Problem pr;
    if (make_problem(pr, N, C, H, W, K, R, S, stride_h, stride_w, pad_h, pad_w, groups, dtype) != MICONV_OK) return "none";
    switch (choose_algo(pass, pr)) {
        case MICONV_ALGO_DIRECT: return "direct";
        case MICONV_ALGO_MFMA: return miconv::mfma_path_name(pass, pr);
        case MICONV_ALGO_DEPTHWISE: return miconv::depthwise_path_name(pass, pr);
        default: return "none";
    }
}

int miconv_set_algo(int pass, int algo) {
    if (pass < 0 || pass > 2) return record_error(MICONV_ERR_DTYPE, "unknown pass %d", pass);
    if (algo < MICONV_ALGO_AUTO || algo > MICONV_ALGO_DEPTHWISE) return record_error(MICONV_ERR_DTYPE, "unknown algorithm %d", algo);
    g_forced[pass] = algo;
    return MICONV_OK;
}

int miconv_last_algo(int pass) {
    if (pass < 0 || pass > 2) return MICONV_ALGO_AUTO;
    return g_last_algo[pass];
}

const char* miconv_last_error(void) { return g_err; }

}  // extern "C"
