// Host side of the tiled forward / stride-1 backward-data path: which instantiation of the kernel in
// mfma_tile_kernel.h serves which filter size and stride.
#include "mfma_tile_kernel.h"

namespace miconv {
namespace {
using namespace tile;

// Two patch buffers everywhere: a third one lets the first LDS operands of the next chunk be requested before the
// barrier, but the shorter start-up and the smaller LDS footprint of two were worth more on every layer measured
// (1-4 %; 1x1 at stride 2 and on 7 x 7 planes 5-7 %).
// XWONLY: the caller has checked that the patch is a run of full rows of an aligned plane, so only that instance is built.
template <typename T, int R, int S, int ST, int TH, int TW, int CK, int WF, int WP, bool BWD, int NBUF = 2, bool PERSIST = false,
          bool XWONLY = false>
hipError_t launch_tile(const TileArgs& base, hipStream_t st) {
    TileArgs a = base;
    a.tiles_h = (a.OH + TH - 1) / TH;
    a.tiles_w = (a.OW + TW - 1) / TW;
    a.fblocks = (a.Fg + 16 * WF - 1) / (16 * WF);
    a.units = a.N * a.groups * a.tiles_h * a.tiles_w;
    a.items = ((a.units + 7) / 8) * 8 * a.fblocks;
    // persistent: one workgroup per CU walks its share of the items
    const int grid = PERSIST && a.items > 256 ? 256 : a.items;
    const bool wv = a.Rg % (CK / 4) == 0 && a.Rg % 4 == 0;   // forward filters can be read four values at a time
    if constexpr (R == 1 && S == 1 && ST == 1 && sizeof(T) == 4 && (TH * TW) % 4 == 0) {
        // patch == plane: contiguous chunks, 16 bytes per lane
        // (a ragged last band reads rows of the next channel or zeros past the tensor; those pixels are not stored)
        const bool plane_patch = a.pad_h == 0 && a.pad_w == 0 && a.IW == TW && a.OW == TW && a.IH == a.OH &&
                                 (a.IH * a.IW) % 4 == 0 && reinterpret_cast<uintptr_t>(a.src) % 16 == 0;
        if (plane_patch) {
            if (wv) conv_tile_kernel<T, R, S, ST, TH, TW, CK, WF, WP, BWD, true, false, NBUF, true, PERSIST><<<grid, 64 * WF * WP, 0, st>>>(a);
            else conv_tile_kernel<T, R, S, ST, TH, TW, CK, WF, WP, BWD, false, false, NBUF, true, PERSIST><<<grid, 64 * WF * WP, 0, st>>>(a);
            return hipGetLastError();
        }
    }
    if constexpr (XWONLY) return hipErrorNotSupported;
    else if (wv) conv_tile_kernel<T, R, S, ST, TH, TW, CK, WF, WP, BWD, true, false, NBUF, false, PERSIST><<<grid, 64 * WF * WP, 0, st>>>(a);
    else conv_tile_kernel<T, R, S, ST, TH, TW, CK, WF, WP, BWD, false, false, NBUF, false, PERSIST><<<grid, 64 * WF * WP, 0, st>>>(a);
    return hipGetLastError();
}

// Picks the instantiation for a filter size / stride.  Returns false when none fits.
template <typename T, bool BWD>
bool dispatch_tile(int R, int S, int stride, const TileArgs& a, hipStream_t st, bool dry, hipError_t* err) {
    *err = hipSuccess;
    if (R == 3 && S == 3 && stride == 1) {
        // eight waves: two per SIMD, so one wave's LDS and barrier waits are covered by the other's MFMAs
        if (dry) return true;
        // planes of at most 7 x 7 pixels: a 7 x 7 tile is 4 pixel blocks (a 14 x 14 tile would run 13 for 3.06)
        if (a.OH <= 7 && a.OW <= 7) {
            // (128 filters per workgroup where the layer has them: 512 channels, N=64: 174 / 134 -> 137 / 113 us)
            if (a.Fg >= 128) *err = launch_tile<T, 3, 3, 1, 7, 7, 16, 8, 1, BWD>(a, st);
            else *err = launch_tile<T, 3, 3, 1, 7, 7, 16, 4, 2, BWD>(a, st);
            return true;
        }
        // Few chunks per item and many items: persistent workgroups hide each item's start-up and write-out
        const long long ids = (long long)a.N * a.groups * ((a.OH + 13) / 14) * ((a.OW + 13) / 14) * ((a.Fg + 63) / 64);
        // Wide planes take 12 x 16 tiles: 12 pixel blocks without a ragged one (14 x 14 = 12.25 blocks run as 13), and
        // output rows of 64 bytes that start on 64-byte boundaries
        // (with 128 filters per workgroup where the layer has them: 64 -> 128 channels at 112 x 112, N=32: 500 -> 476 us)
        if (a.Fg >= 128 && a.Rg <= 128 && ids >= 1024 && a.OW % 16 == 0 && a.OH >= 96) *err = launch_tile<T, 3, 3, 1, 12, 16, 16, 8, 1, BWD, 2, true>(a, st);
        else if (a.Rg <= 128 && ids >= 1024 && a.OW % 16 == 0 && a.OH >= 96) *err = launch_tile<T, 3, 3, 1, 12, 16, 16, 4, 2, BWD, 2, true>(a, st);
        else if (a.Rg <= 128 && ids >= 1024) *err = launch_tile<T, 3, 3, 1, 14, 14, 16, 4, 2, BWD, 2, true>(a, st);
        // 128 filters per workgroup (eight waves x 16 filters x all 13 pixel blocks) where that leaves a workgroup for
        // every CU: the patch is fetched and stored to LDS once per 128 filters and a wave's filter values are used 12.25
        // times (512 channels at 28 x 28, N=64: 1679 / 1657 -> 1606 / 1596 us; 256 channels at 56 x 56, N=32: 871 -> 823 us)
        else if (a.Fg >= 128 && ids >= 512) *err = launch_tile<T, 3, 3, 1, 14, 14, 16, 8, 1, BWD, 2>(a, st);
        else *err = launch_tile<T, 3, 3, 1, 14, 14, 16, 4, 2, BWD, 2>(a, st);
        return true;
    }
    if (R == 1 && S == 1 && stride == 1) {
        if (dry) return true;
        // 32-channel chunks on eight waves (64-channel chunks leave one workgroup per CU: 80 instead of 68 us on
        // the 1024 -> 256 channel layer); persistent workgroups when there are many short items
        if (a.OH <= 7 && a.OW <= 7) {
            // 128 filters per workgroup where the layer has them: each of the eight waves then runs the plane's three full
            // pixel blocks and the one-pixel block (512 <-> 2048 channels, N=64: 72-79 -> 62-64 us)
            if (a.Fg >= 128) *err = launch_tile<T, 1, 1, 1, 7, 7, 32, 8, 1, BWD>(a, st);
            else *err = launch_tile<T, 1, 1, 1, 7, 7, 32, 4, 2, BWD>(a, st);
            return true;
        }
        // planes 28, 56 or 112 pixels wide: bands of full rows, 224 pixels = 14 blocks, fetched 16 bytes per lane; two
        // patch buffers, so that two workgroups share a CU
        if constexpr (sizeof(T) == 4) {
            if (a.pad_h == 0 && a.pad_w == 0 && a.IH == a.OH && a.IW == a.OW && (a.OW == 28 || a.OW == 56 || a.OW == 112) &&
                reinterpret_cast<uintptr_t>(a.src) % 16 == 0) {
                // 128 filters per workgroup where the layer has them (3-7 %)
                if (a.Fg >= 128) {
                    if (a.OW == 28) *err = launch_tile<T, 1, 1, 1, 8, 28, 32, 8, 1, BWD, 2, true, true>(a, st);
                    else if (a.OW == 56) *err = launch_tile<T, 1, 1, 1, 4, 56, 32, 8, 1, BWD, 2, true, true>(a, st);
                    else *err = launch_tile<T, 1, 1, 1, 2, 112, 32, 8, 1, BWD, 2, true, true>(a, st);
                    return true;
                }
                if (a.OW == 28) *err = launch_tile<T, 1, 1, 1, 8, 28, 32, 4, 2, BWD, 2, true, true>(a, st);
                else if (a.OW == 56) *err = launch_tile<T, 1, 1, 1, 4, 56, 32, 4, 2, BWD, 2, true, true>(a, st);
                else *err = launch_tile<T, 1, 1, 1, 2, 112, 32, 4, 2, BWD, 2, true, true>(a, st);
                return true;
            }
        }
        const long long ids = (long long)a.N * a.groups * ((a.OH + 13) / 14) * ((a.OW + 13) / 14) * ((a.Fg + 63) / 64);
        // 128 filters per workgroup (eight waves x 16 filters x all 13 pixel blocks) where that still leaves two
        // workgroups per CU: a chunk then lasts twice as long against the same patch traffic, and a wave's filter values are
        // used 12.25 times instead of 6 (512 -> 512 channels, N=128: forward 117 -> 106 us, backward-data 119 -> 107 us;
        // 256 -> 1024 channels backward-data, N=64: 68 -> 62 us)
        const long long ids128 = (long long)a.N * a.groups * ((a.OH + 13) / 14) * ((a.OW + 13) / 14) * ((a.Fg + 127) / 128);
        if (ids128 >= 512 && (a.Fg % 128 == 0 || a.Fg >= 512)) {
            *err = launch_tile<T, 1, 1, 1, 14, 14, 32, 8, 1, BWD, 2>(a, st);
            return true;
        }
        if (a.Rg <= 256 && ids >= 1024) *err = launch_tile<T, 1, 1, 1, 14, 14, 32, 4, 2, BWD, 2, true>(a, st);
        else *err = launch_tile<T, 1, 1, 1, 14, 14, 32, 4, 2, BWD, 2>(a, st);
        return true;
    }
    if (!BWD && R == 1 && S == 1 && stride == 2) {
        // the 1x1 stride-2 shortcut of a residual network: every other pixel of every other row
        if (dry) return true;
        // (128 filters per workgroup: 256 -> 512 channels, 56 -> 28, N=64: 182 -> 145 us)
        if (a.Fg >= 128) *err = launch_tile<T, 1, 1, 2, 14, 14, 32, 8, 1, false>(a, st);
        else *err = launch_tile<T, 1, 1, 2, 14, 14, 32, 4, 2, false>(a, st);
        return true;
    }
    if (!BWD && R == 3 && S == 3 && stride == 2) {
        if (dry) return true;
        // 64 filters x 14 x 14 pixels per workgroup unless that leaves CUs without one; then half tiles (7 x 14) on twice
        // the workgroups, eight waves and two patch buffers (128 -> 128 channels, 28 -> 14, N=64: 40.2 -> 37.2 us; with
        // 32 filters x 14 x 14 pixels every workgroup fetched the whole patch for half of the MFMAs), and only when
        // that is still too few, 32 filters per workgroup
        const long long wgs64 = (long long)a.N * a.groups * ((a.OH + 13) / 14) * ((a.OW + 13) / 14) * ((a.Fg + 63) / 64);
        const long long wgs64h = (long long)a.N * a.groups * ((a.OH + 6) / 7) * ((a.OW + 13) / 14) * ((a.Fg + 63) / 64);
        if (wgs64 >= 200) *err = launch_tile<T, 3, 3, 2, 14, 14, 8, 4, 1, false>(a, st);
        else if (wgs64h >= 200) *err = launch_tile<T, 3, 3, 2, 7, 14, 8, 4, 2, false, 2>(a, st);
        else *err = launch_tile<T, 3, 3, 2, 14, 14, 8, 2, 4, false, 2>(a, st);
        return true;
    }
    return false;
}

// Builds the operand view of a pass; false when the tiled kernel cannot run it.
bool make_args(int pass, const Problem& pr, const void* in0, const void* in1, float* out, TileArgs& a, int& stride) {
    if (pr.sh != pr.sw) return false;
    // Buffer descriptors address at most 2 GiB here.
    const size_t esz = pr.dtype == 0 ? 4 : 2;
    const size_t lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    const unsigned wbytes = (unsigned)((size_t)pr.K * pr.Cg * pr.R * pr.S * esz);
    if (pass == 0) {
        a = TileArgs{in0, in1, out, pr.N, pr.C, pr.H, pr.W, pr.K, pr.P, pr.Q, pr.Kg, pr.Cg, pr.groups,
                     pr.ph, pr.pw, 0, 0, 0, 0, wbytes};
        a.bias = pr.bias;
        stride = pr.sh;
        return true;
    }
    if (pass == 1) {
        if (pr.sh != 1) return false;
        a = TileArgs{in0, in1, out, pr.N, pr.K, pr.P, pr.Q, pr.C, pr.H, pr.W, pr.Cg, pr.Kg, pr.groups,
                     pr.R - 1 - pr.ph, pr.S - 1 - pr.pw, 0, 0, 0, 0, wbytes};
        a.mask = pr.relu_mask;
        stride = 1;
        return true;
    }
    return false;
}

}  // namespace

bool tile_supports(int pass, const Problem& pr) {
    TileArgs a;
    int stride;
    hipError_t e;
    if (!make_args(pass, pr, nullptr, nullptr, nullptr, a, stride)) return false;
    return pass == 0 ? dispatch_tile<float, false>(pr.R, pr.S, stride, a, nullptr, true, &e)
                     : dispatch_tile<float, true>(pr.R, pr.S, stride, a, nullptr, true, &e);
}

hipError_t tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, hipStream_t st) {
    TileArgs a;
    int stride;
    hipError_t e = hipErrorNotSupported;
    if (!make_args(pass, pr, in0, in1, out, a, stride)) return e;
    bool ok;
    if (pr.dtype == 0)
        ok = pass == 0 ? dispatch_tile<float, false>(pr.R, pr.S, stride, a, st, false, &e)
                       : dispatch_tile<float, true>(pr.R, pr.S, stride, a, st, false, &e);
    else
        ok = pass == 0 ? dispatch_tile<uint16_t, false>(pr.R, pr.S, stride, a, st, false, &e)
                       : dispatch_tile<uint16_t, true>(pr.R, pr.S, stride, a, st, false, &e);
    return ok ? e : hipErrorNotSupported;
}

}  // namespace miconv
