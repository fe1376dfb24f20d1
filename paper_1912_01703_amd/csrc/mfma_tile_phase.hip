// Backward-data for stride > 1 on the tiled MFMA kernel: one launch per output phase, or (3x3, stride 2,
// padding 1) one launch in which all four phases share the dy patch.
//
//   dx[n,c,h,v] = sum_{k,r,s : (h+ph-r) % st == 0, (v+pw-s) % st == 0} dy[n,k,(h+ph-r)/st,(v+pw-s)/st] * w[k,c,r,s]
//
// Only the taps r congruent to (h+ph) modulo the stride can reach row h, so the rows with
// (h+ph) % st == a (a "phase") form an independent problem: with h = st*i + a - ph and r = a + st*j,
//   dx_a[i] = sum_j dy[i - j] * w[a + st*j],        j = 0 .. J_a-1,  J_a = ceil((R - a) / st),
// a stride-1 correlation of dy with the J_a taps taken in reverse.  The same holds for columns, so a
// stride-st backward pass is st*st stride-1 problems with sub-filters of J_a x J_b taps whose outputs
// interleave in dx.  Gathering dy with zero-stuffing instead would spend st*st times the MFMA work on
// structural zeros.  Phases without any tap (filter smaller than the stride, e.g. a 1x1 stride-2 shortcut) leave
// zeros in dx: dx is cleared by a fill kernel first (no memset node: callers may capture the stream).
#include "mfma_tile_kernel.h"

namespace miconv {
namespace {
using namespace tile;

struct Phase {
    int J;    // taps
    int i0;   // first phase-grid index whose row lies inside the image
    int cnt;  // rows of dx in this phase
};

// Rows h in [0, H) with (h + pad) % st == a are h = st*i + a - pad for i = i0 .. i0+cnt-1.
Phase make_phase(int a, int st, int R, int pad, int H) {
    Phase p;
    p.J = a < R ? (R - a + st - 1) / st : 0;
    const int lo = pad - a;                       // need st*i >= lo
    p.i0 = lo <= 0 ? 0 : (lo + st - 1) / st;
    const int hi = H - 1 + pad - a;               // need st*i <= hi
    p.cnt = hi < 0 ? 0 : hi / st - p.i0 + 1;
    if (p.cnt < 0) p.cnt = 0;
    return p;
}

// WF x WP waves: 4 x 1 (64 destination channels per workgroup), 2 x 4 for small grids or, when the layer
// has at most 16 destination channels per group (backward-data of a first layer), 1 x 4 so that no wave is idle.
template <typename T, int JH, int JW, int WF, int WP>
hipError_t launch_phase_waves(TileArgs a, hipStream_t st) {
    constexpr int TH = 14, TW = 14, CK = 16;
    a.tiles_h = (a.OH + TH - 1) / TH;
    a.tiles_w = (a.OW + TW - 1) / TW;
    a.fblocks = (a.Fg + 16 * WF - 1) / (16 * WF);
    a.units = a.N * a.groups * a.tiles_h * a.tiles_w;
    a.items = ((a.units + 7) / 8) * 8 * a.fblocks;
    const int grid = a.items;
    conv_tile_kernel<T, JH, JW, 1, TH, TW, CK, WF, WP, true, false, true, 2><<<grid, 64 * WF * WP, 0, st>>>(a);
    return hipGetLastError();
}

template <typename T, int JH, int JW>
hipError_t launch_phase(const TileArgs& a, hipStream_t st) {
    if (a.Fg <= 16) return launch_phase_waves<T, JH, JW, 1, 4>(a, st);
    // 64 destination channels per workgroup unless that leaves CUs without one; then 32 on twice the workgroups
    const long long wgs64 = (long long)a.N * a.groups * ((a.OH + 13) / 14) * ((a.OW + 13) / 14) * ((a.Fg + 63) / 64);
    // 128 destination channels on eight waves where that leaves two workgroups per CU (1x1, 512 -> 256 channels, 28 -> 56, N=64: 163 -> 145 us)
    if (a.Fg >= 128 && wgs64 >= 1024) return launch_phase_waves<T, JH, JW, 8, 1>(a, st);
    return wgs64 >= 200 ? launch_phase_waves<T, JH, JW, 4, 1>(a, st) : launch_phase_waves<T, JH, JW, 2, 4>(a, st);
}

template <typename T>
hipError_t launch_phase_shape(int jh, int jw, const TileArgs& a, hipStream_t st) {
    switch (jh * 10 + jw) {
        case 11: return launch_phase<T, 1, 1>(a, st);
        case 12: return launch_phase<T, 1, 2>(a, st);
        case 13: return launch_phase<T, 1, 3>(a, st);
        case 21: return launch_phase<T, 2, 1>(a, st);
        case 22: return launch_phase<T, 2, 2>(a, st);
        case 23: return launch_phase<T, 2, 3>(a, st);
        case 31: return launch_phase<T, 3, 1>(a, st);
        case 32: return launch_phase<T, 3, 2>(a, st);
        case 33: return launch_phase<T, 3, 3>(a, st);
        default: return hipErrorNotSupported;
    }
}

// 3x3, stride 2, padding 1: the merged kernel (MERGE2 in mfma_tile_kernel.h).
template <typename T, int WF, int WP, int TH = 14, int NBUF = 2>
hipError_t launch_merge2(TileArgs a, hipStream_t st) {
    constexpr int TW = 14, CK = 16;
    a.tiles_h = (a.OH + TH - 1) / TH;
    a.tiles_w = (a.OW + TW - 1) / TW;
    a.fblocks = (a.Fg + 16 * WF - 1) / (16 * WF);
    a.units = a.N * a.groups * a.tiles_h * a.tiles_w;
    a.items = ((a.units + 7) / 8) * 8 * a.fblocks;
    conv_tile_kernel<T, 3, 3, 1, TH, TW, CK, WF, WP, true, false, false, NBUF, false, false, true><<<a.items, 64 * WF * WP, 0, st>>>(a);
    return hipGetLastError();
}

__global__ __launch_bounds__(256) void zero_fill_kernel(float* __restrict__ dst, size_t count) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i + 4 <= count && reinterpret_cast<uintptr_t>(dst) % 16 == 0) {
        *reinterpret_cast<float4*>(dst + i) = make_float4(0.f, 0.f, 0.f, 0.f);
    } else {
        for (size_t j = i; j < count && j < i + 4; ++j) dst[j] = 0.f;
    }
}

bool merge2_ok(const Problem& pr) {
    if (pr.R != 3 || pr.S != 3 || pr.sh != 2 || pr.sw != 2 || pr.ph != 1 || pr.pw != 1) return false;
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    return (size_t)pr.N * pr.C * pr.H * pr.W * esz < lim && (size_t)pr.N * pr.K * pr.P * pr.Q * esz < lim;
}

}  // namespace

bool tile_merge2_supports(const Problem& pr) { return merge2_ok(pr); }

hipError_t tile_merge2_run(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st) {
    if (!merge2_ok(pr)) return hipErrorNotSupported;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    TileArgs t{};
    t.src = dy; t.wgt = w; t.dst = dx;
    t.N = pr.N; t.Csrc = pr.K; t.IH = pr.P; t.IW = pr.Q;
    t.Cdst = pr.C; t.OH = (pr.H + 1) / 2; t.OW = (pr.W + 1) / 2;   // the half-resolution grid
    t.Fg = pr.Cg; t.Rg = pr.Kg; t.groups = pr.groups;
    t.pad_h = 0; t.pad_w = 0;                                     // patch row 0 is dy row (grid row of the tile)
    t.wgt_bytes = (unsigned)((size_t)pr.K * pr.Cg * pr.R * pr.S * esz);
    t.DH = pr.H; t.DW = pr.W;
    t.w_rs = 9;
    t.mask = pr.relu_mask;
    if (t.Fg <= 16) return pr.dtype == 0 ? launch_merge2<float, 1, 4>(t, st) : launch_merge2<uint16_t, 1, 4>(t, st);
    // 64 destination channels x 7 x 14 grid positions on eight waves with two patch buffers where the channels fill such
    // blocks (128 channels, 28 x 28, N=64: 42.4 -> 40.6 us; 256 channels: 137 -> 131 us), else 32 channels x 14 x 14
    if (t.Fg % 64 == 0 || t.Fg >= 256)
        return pr.dtype == 0 ? launch_merge2<float, 4, 2, 7>(t, st) : launch_merge2<uint16_t, 4, 2, 7>(t, st);
    return pr.dtype == 0 ? launch_merge2<float, 2, 4>(t, st) : launch_merge2<uint16_t, 2, 4>(t, st);
}

bool tile_phase_supports(const Problem& pr) {
    if (pr.sh < 2 && pr.sw < 2) return false;   // stride 1 runs on the plain path
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    for (int a = 0; a < pr.sh; ++a) {
        const Phase p = make_phase(a, pr.sh, pr.R, pr.ph, pr.H);
        if (p.cnt > 0 && p.J > 3) return false;
    }
    for (int b = 0; b < pr.sw; ++b) {
        const Phase p = make_phase(b, pr.sw, pr.S, pr.pw, pr.W);
        if (p.cnt > 0 && p.J > 3) return false;
    }
    return true;
}

hipError_t tile_phase_run(const Problem& pr, const void* dy, const void* w, float* dx, hipStream_t st) {
    if (!tile_phase_supports(pr)) return hipErrorNotSupported;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    bool empty = false;   // a phase that no tap reaches
    for (int a = 0; a < pr.sh; ++a) empty |= make_phase(a, pr.sh, pr.R, pr.ph, pr.H).J == 0;
    for (int b = 0; b < pr.sw; ++b) empty |= make_phase(b, pr.sw, pr.S, pr.pw, pr.W).J == 0;
    // 1x1 at stride 2 without padding: the kernel writes the zeros of the three empty phases next to its results
    const bool fill2 = pr.R == 1 && pr.S == 1 && pr.sh == 2 && pr.sw == 2 && pr.ph == 0 && pr.pw == 0;
    if (empty && !fill2) {
        const size_t count = (size_t)pr.N * pr.C * pr.H * pr.W;
        zero_fill_kernel<<<(unsigned)((count / 4 + 256) / 256), 256, 0, st>>>(dx, count);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int a = 0; a < pr.sh; ++a) {
        const Phase ph = make_phase(a, pr.sh, pr.R, pr.ph, pr.H);
        if (ph.cnt == 0 || ph.J == 0) continue;
        for (int b = 0; b < pr.sw; ++b) {
            const Phase pw = make_phase(b, pr.sw, pr.S, pr.pw, pr.W);
            if (pw.cnt == 0 || pw.J == 0) continue;
            TileArgs t{};
            t.src = dy; t.wgt = w; t.dst = dx;
            t.N = pr.N; t.Csrc = pr.K; t.IH = pr.P; t.IW = pr.Q;
            t.Cdst = pr.C; t.OH = ph.cnt; t.OW = pw.cnt;
            t.Fg = pr.Cg; t.Rg = pr.Kg; t.groups = pr.groups;
            // local output o = i - i0 reads dy rows o + i0 - (J-1) + j', j' = 0 .. J-1
            t.pad_h = ph.J - 1 - ph.i0; t.pad_w = pw.J - 1 - pw.i0;
            t.wgt_bytes = (unsigned)((size_t)pr.K * pr.Cg * pr.R * pr.S * esz);
            t.o_sh = pr.sh; t.o_sw = pr.sw;
            t.o_oh = pr.sh * ph.i0 + a - pr.ph; t.o_ow = pr.sw * pw.i0 + b - pr.pw;
            t.DH = pr.H; t.DW = pr.W;
            t.w_rs = pr.R * pr.S;
            t.mask = pr.relu_mask;
            t.fill2 = fill2 ? (pr.W % 2 == 0 && reinterpret_cast<uintptr_t>(dx) % 8 == 0 ? 2 : 1) : 0;
            for (int jr = 0; jr < ph.J; ++jr)
                for (int js = 0; js < pw.J; ++js)
                    t.tapoff[jr * pw.J + js] = (a + pr.sh * (ph.J - 1 - jr)) * pr.S + (b + pr.sw * (pw.J - 1 - js));
            const hipError_t e = pr.dtype == 0 ? launch_phase_shape<float>(ph.J, pw.J, t, st)
                                               : launch_phase_shape<uint16_t>(ph.J, pw.J, t, st);
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace miconv
