// Depthwise convolution (groups == C == K): every channel is a single-plane 3x3
// stencil, 18 FLOP per 8 bytes moved, so all three passes are bound by HBM
// bandwidth and use no MFMA.  The kernels move each input byte from global
// memory exactly once, as coalesced runs of whole image rows, into a
// zero-bordered copy of the plane in LDS, and do all tap reuse from LDS.
//
//   forward        y[n,c,p,q]  = sum_{r,s} x[n,c,p*st-ph+r,q*st-pw+s] * w[c,0,r,s]
//   backward-data  dx[n,c,h,v] = sum_{r,s} dy[n,c,h+ph-r,v+pw-s] * w[c,0,r,s]        (stride 1: the same
//                  stencil on dy with the filter rotated by 180 degrees and padding R-1-ph)
//   backward-weight dw[c,0,r,s] = sum_{n,p,q} dy[n,c,p,q] * x[n,c,p*st-ph+r,q*st-pw+s]
//
// Planes of consecutive channels (and images) are adjacent in memory, so a
// workgroup takes a batch of PL consecutive planes: one contiguous region.
// Index arithmetic uses multiplication by a float reciprocal (exact for the
// small ranges involved: the fractional part of (e+0.5)/d is at least 0.5/d
// away from an integer, far more than fp32 rounding) instead of integer division.
#include "common.h"

namespace miconv {
namespace {

constexpr int kThreads = 256;

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
__device__ __forceinline__ int fdiv(int e, float inv) { return (int)(((float)e + 0.5f) * inv); }

struct DwArgs {
    const void* src;   // x (forward) or dy (backward-data)
    const void* w;
    float* dst;
    int planes, C;     // N*C planes; channel of plane i is i % C
    int IH, IW, OH, OW;
    int pad_h, pad_w;  // source row = out row * ST - pad_h + r
    int PL;            // planes per workgroup
    int PPH, PPW;      // padded plane held in LDS
    float inv_ppw, inv_pps, inv_ow, inv_g4;
    int G4;            // groups of 4 consecutive outputs per plane
    int vec;           // outputs of a group may be stored as one float4
    int flip;          // rotate the filter by 180 degrees (backward-data)
};

// LDS: [PL][PPH*PPW] source planes with zero borders, then [PL][R*S] filters.
template <typename T, int R, int S, int ST>
__global__ __launch_bounds__(kThreads) void dw_stencil_kernel(DwArgs a) {
    extern __shared__ float lds[];
    constexpr int RS = R * S;
    const int tid = threadIdx.x;
    const int PPS = a.PPH * a.PPW;
    const int plane0 = blockIdx.x * a.PL;
    const int np = min(a.PL, a.planes - plane0);
    const int iplane = a.IH * a.IW, oplane = a.OH * a.OW;
    const T* const tnull = nullptr;
    float* wl = lds + a.PL * PPS;

    // ---- stage the batch: one contiguous region of np planes, gathered into padded planes ----------
    const rsrc_t srs = make_rsrc(static_cast<const T*>(a.src) + (size_t)plane0 * iplane,
                                 (unsigned)(np * iplane) * (unsigned)sizeof(T));
    const int total = a.PL * PPS;
    for (int e = tid; e < total; e += kThreads) {
        const int pl = fdiv(e, a.inv_pps);
        const int rem = e - pl * PPS;
        const int ph = fdiv(rem, a.inv_ppw);
        const int pw = rem - ph * a.PPW;
        const int ih = ph - a.pad_h, iw = pw - a.pad_w;
        const bool ok = ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;   // planes past np fall outside the descriptor
        lds[e] = buf_load(srs, ok ? (unsigned)(pl * iplane + ih * a.IW + iw) * (unsigned)sizeof(T) : kOob, tnull);
    }
    const rsrc_t wrs = make_rsrc(a.w, (unsigned)(a.C * RS) * (unsigned)sizeof(T));
    for (int e = tid; e < a.PL * RS; e += kThreads) {
        const int pl = e / RS, t = e - pl * RS;
        const int c = (plane0 + pl) % a.C;
        wl[e] = buf_load(wrs, pl < np ? (unsigned)(c * RS + (a.flip ? RS - 1 - t : t)) * (unsigned)sizeof(T) : kOob, tnull);
    }
    __syncthreads();

    // ---- stencil: one item = 4 consecutive outputs of one plane --------------------------------------
    const int items = np * a.G4;
    float* dst = a.dst + (size_t)plane0 * oplane;
    for (int it = tid; it < items; it += kThreads) {
        const int pl = fdiv(it, a.inv_g4);
        const int j0 = 4 * (it - pl * a.G4);
        const float* xp = lds + pl * PPS;
        float wv[RS];
#pragma unroll
        for (int t = 0; t < RS; ++t) wv[t] = wl[pl * RS + t];
        float out[4];
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            int j = j0 + o;
            if (j >= oplane) j = oplane - 1;   // ragged last group: computed, not stored
            const int p = fdiv(j, a.inv_ow);
            const int q = j - p * a.OW;
            const float* xq = xp + p * ST * a.PPW + q * ST;
            float acc = 0.f;
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s = 0; s < S; ++s) acc = fmaf(xq[r * a.PPW + s], wv[r * S + s], acc);
            out[o] = acc;
        }
        float* d = dst + (size_t)pl * oplane + j0;
        if (a.vec) {
            *reinterpret_cast<float4*>(d) = make_float4(out[0], out[1], out[2], out[3]);
        } else {
#pragma unroll
            for (int o = 0; o < 4; ++o)
                if (j0 + o < oplane) d[o] = out[o];
        }
    }
}

// ---- backward-weight ------------------------------------------------------------------------------
// A workgroup owns PL consecutive channels and a contiguous range of images.  Thread items are
// (channel, group of 4 output pixels) and stay the same for every image, so the R*S partial sums
// live in registers across the image loop; they are combined per channel through LDS in a fixed
// order and written to dw (one split) or to a partial buffer summed afterwards in split order.
struct DwWArgs {
    const void* x;
    const void* dy;
    float* out;        // dw or partial buffer [nsplit][C*R*S]
    int N, C, H, W, P, Q;
    int pad_h, pad_w;
    int PL, PPH, PPW;
    float inv_ppw, inv_pps, inv_q, inv_g4;
    int G4;
    int cblocks, nsplit;
};

template <typename T, int R, int S, int ST, int IPT>
__global__ __launch_bounds__(kThreads) void dw_wgrad_kernel(DwWArgs a) {
    extern __shared__ float lds[];
    constexpr int RS = R * S;
    const int tid = threadIdx.x;
    const int PPS = a.PPH * a.PPW;
    const int cb = blockIdx.x % a.cblocks, sp = blockIdx.x / a.cblocks;
    const int c0 = cb * a.PL;
    const int np = min(a.PL, a.C - c0);
    const int n_begin = (int)((long long)a.N * sp / a.nsplit), n_end = (int)((long long)a.N * (sp + 1) / a.nsplit);
    const int xplane = a.H * a.W, yplane = a.P * a.Q;
    const T* const tnull = nullptr;
    float* xl = lds;                  // [PL][PPS]
    float* yl = lds + a.PL * PPS;     // [PL][P*Q]

    // per-thread items: fixed for the whole image loop
    const int items = np * a.G4;
    int xo[IPT][4], yo[IPT], j0a[IPT];
    bool live[IPT];
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int it = tid + kThreads * i;
        live[i] = it < items;
        const int itc = live[i] ? it : 0;
        const int pl = fdiv(itc, a.inv_g4);
        const int j0 = 4 * (itc - pl * a.G4);
        yo[i] = pl * yplane + j0;
        j0a[i] = j0;
#pragma unroll
        for (int o = 0; o < 4; ++o) {
            int j = j0 + o;
            if (j >= yplane) j = yplane - 1;
            const int p = fdiv(j, a.inv_q), q = j - p * a.Q;
            xo[i][o] = pl * PPS + p * ST * a.PPW + q * ST;
        }
    }
    float acc[IPT][RS];
#pragma unroll
    for (int i = 0; i < IPT; ++i)
#pragma unroll
        for (int t = 0; t < RS; ++t) acc[i][t] = 0.f;

    for (int n = n_begin; n < n_end; ++n) {
        const rsrc_t xrs = make_rsrc(static_cast<const T*>(a.x) + ((size_t)n * a.C + c0) * xplane,
                                     (unsigned)(np * xplane) * (unsigned)sizeof(T));
        const rsrc_t yrs = make_rsrc(static_cast<const T*>(a.dy) + ((size_t)n * a.C + c0) * yplane,
                                     (unsigned)(np * yplane) * (unsigned)sizeof(T));
        for (int e = tid; e < a.PL * PPS; e += kThreads) {
            const int pl = fdiv(e, a.inv_pps);
            const int rem = e - pl * PPS;
            const int ph = fdiv(rem, a.inv_ppw);
            const int pw = rem - ph * a.PPW;
            const int ih = ph - a.pad_h, iw = pw - a.pad_w;
            const bool ok = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            xl[e] = buf_load(xrs, ok ? (unsigned)(pl * xplane + ih * a.W + iw) * (unsigned)sizeof(T) : kOob, tnull);
        }
        for (int e = tid; e < a.PL * yplane; e += kThreads)
            yl[e] = buf_load(yrs, (unsigned)e * (unsigned)sizeof(T), tnull);   // past np planes: zero
        __syncthreads();
#pragma unroll
        for (int i = 0; i < IPT; ++i) {
            if (!live[i]) continue;
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                // the ragged tail of a plane's last group multiplies by zero
                const bool in_plane = j0a[i] + o < yplane;
                const float g = in_plane ? yl[yo[i] + o] : 0.f;
                const float* xq = xl + xo[i][o];
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int s = 0; s < S; ++s) acc[i][r * S + s] = fmaf(g, xq[r * a.PPW + s], acc[i][r * S + s]);
            }
        }
        __syncthreads();
    }

    // ---- per-channel sum over the G4 items, fixed order: item partials to LDS, then one thread per (channel, tap)
    float* red = lds;   // [items][RS], fits: items*RS <= PL*G4*RS floats (checked on the host)
#pragma unroll
    for (int i = 0; i < IPT; ++i)
        if (live[i])
#pragma unroll
            for (int t = 0; t < RS; ++t) red[(tid + kThreads * i) * RS + t] = acc[i][t];
    __syncthreads();
    float* out = a.out + (a.nsplit > 1 ? (size_t)sp * a.C * RS : 0);
    for (int e = tid; e < np * RS; e += kThreads) {
        const int pl = e / RS, t = e - pl * RS;
        float sum = 0.f;
        for (int gidx = 0; gidx < a.G4; ++gidx) sum += red[(pl * a.G4 + gidx) * RS + t];
        out[(size_t)(c0 + pl) * RS + t] = sum;
    }
}

__global__ __launch_bounds__(256) void dw_reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                               int nsplit, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = part[i];
    for (int s = 1; s < nsplit; ++s) sum += part[(size_t)s * count + i];
    dw[i] = sum;
}

// ====================================================================================================
// Wave-private variants for small planes (the usual depthwise shapes: 7x7 ... 28x28).
// A wave owns whole planes: it fetches PB planes at once (PB*NPI loads in flight per lane), copies
// them into its own zero-bordered LDS region and computes them, so there is no workgroup barrier at
// all and every quantity that depends only on the lane (gather offsets, LDS offsets of the four
// outputs a lane produces) is computed once per kernel instead of once per element.
// ====================================================================================================
struct DwWaveArgs {
    const void* src;
    const void* w;
    float* dst;
    int planes, C;
    int IH, IW, OH, OW, pad_h, pad_w;
    int PPH, PPW;
    int NO, LS;        // a lane produces outputs lane + LS*o, o < NO (LS <= 64, NO*LS >= OH*OW)
    float inv_ppw, inv_ow;
    int flip, nbatches;
    unsigned src_bytes;
};

// NPI: 64-lane passes over the padded plane (NPI*64 >= PPH*PPW).  NOM: most outputs per lane.
// PB: planes fetched together.  Consecutive lanes produce consecutive outputs, so LDS reads are
// conflict-free and every store instruction writes one contiguous run.
template <typename T, int ST, int NPI, int NOM, int PB>
__global__ __launch_bounds__(kThreads) void dw_wave_stencil_kernel(DwWaveArgs a) {
    extern __shared__ float lds[];
    constexpr unsigned ESZ = sizeof(T);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform, kept in a scalar register
    const int PPS = a.PPH * a.PPW;
    const int iplane = a.IH * a.IW, oplane = a.OH * a.OW;
    const T* const tnull = nullptr;
    const T* __restrict__ wg = static_cast<const T*>(a.w);
    float* my = lds + wave * PB * PPS;

    unsigned goff[NPI];
#pragma unroll
    for (int i = 0; i < NPI; ++i) {
        const int e = lane + 64 * i;
        const int ph = fdiv(e, a.inv_ppw), pw = e - ph * a.PPW;
        const int ih = ph - a.pad_h, iw = pw - a.pad_w;
        const bool ok = e < PPS && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
        goff[i] = ok ? (unsigned)(ih * a.IW + iw) * ESZ : kOob;
    }
    int xo[NOM];      // LDS offset of the window of output o
    int jo[NOM];      // its index in the output plane, -1 if this lane has no such output
#pragma unroll
    for (int o = 0; o < NOM; ++o) {
        const int j = lane + a.LS * o;
        const bool ok = o < a.NO && lane < a.LS && j < oplane;
        const int jc = ok ? j : 0;
        const int p = fdiv(jc, a.inv_ow), q = jc - p * a.OW;
        xo[o] = p * ST * a.PPW + q * ST;
        jo[o] = ok ? j : -1;
    }

    const rsrc_t srs = make_rsrc(a.src, a.src_bytes);
    const int nw = gridDim.x * (kThreads / 64);
    for (int b = blockIdx.x * (kThreads / 64) + wave; b < a.nbatches; b += nw) {
        const int p0 = b * PB;
        float v[PB][NPI];
        // Planes past the end lie beyond the descriptor (and kOob pushes any offset beyond it): zeros.
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int i = 0; i < NPI; ++i)
                v[pb][i] = buf_load(srs, (unsigned)((p0 + pb) * iplane) * ESZ + goff[i], tnull);
        // The filters of the batch: wave-uniform addresses (scalar loads where the type allows).
        float wv[PB][9];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int pc = p0 + pb < a.planes ? p0 + pb : a.planes - 1;
            const int c = pc % a.C;
#pragma unroll
            for (int t = 0; t < 9; ++t) wv[pb][t] = load_elem(wg, (size_t)(c * 9 + (a.flip ? 8 - t : t)));
        }
#pragma unroll
        for (int pb = 0; pb < PB; ++pb)
#pragma unroll
            for (int i = 0; i < NPI; ++i)
                if (lane + 64 * i < PPS) my[pb * PPS + lane + 64 * i] = v[pb][i];
#pragma unroll
        for (int pb = 0; pb < PB; ++pb) {
            const int plane = p0 + pb;
            if (plane >= a.planes) break;
            const float* xp = my + pb * PPS;
            float* d = a.dst + (size_t)plane * oplane;
#pragma unroll
            for (int o = 0; o < NOM; ++o) {
                if (o >= a.NO) break;
                const float* xq = xp + xo[o];
                float acc = 0.f;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s) acc = fmaf(xq[r * a.PPW + s], wv[pb][r * 3 + s], acc);
                if (jo[o] >= 0) d[jo[o]] = acc;
            }
        }
    }
}

struct DwWaveWArgs {
    const void* x;
    const void* dy;
    float* out;      // [nsplit][C*9] (or dw itself when nsplit == 1)
    int N, C, H, W, P, Q, pad_h, pad_w;
    int PPH, PPW;
    int NO, LS;
    float inv_ppw, inv_q;
    int nsplit;
    unsigned x_bytes, y_bytes;
};

// One wave = one channel and a contiguous range of images.  The nine partial sums of every lane stay
// in registers over the image loop, the next image is fetched while the current one is multiplied,
// and the lanes are combined at the end by a fixed butterfly: bit-reproducible, no atomics.
template <typename T, int ST, int NPI, int NOM>
__global__ __launch_bounds__(kThreads) void dw_wave_wgrad_kernel(DwWaveWArgs a) {
    extern __shared__ float lds[];
    constexpr unsigned ESZ = sizeof(T);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int PPS = a.PPH * a.PPW;
    const int xplane = a.H * a.W, yplane = a.P * a.Q;
    const T* const tnull = nullptr;
    float* my = lds + wave * PPS;
    const int unit = blockIdx.x * (kThreads / 64) + wave;   // = sp * C + c
    if (unit >= a.C * a.nsplit) return;
    const int c = unit % a.C, sp = unit / a.C;
    const int n0 = (int)((long long)a.N * sp / a.nsplit), n1 = (int)((long long)a.N * (sp + 1) / a.nsplit);

    unsigned goff[NPI];
#pragma unroll
    for (int i = 0; i < NPI; ++i) {
        const int e = lane + 64 * i;
        const int ph = fdiv(e, a.inv_ppw), pw = e - ph * a.PPW;
        const int ih = ph - a.pad_h, iw = pw - a.pad_w;
        const bool ok = e < PPS && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        goff[i] = ok ? (unsigned)(ih * a.W + iw) * ESZ : kOob;
    }
    int xo[NOM];
    unsigned yoff[NOM];
#pragma unroll
    for (int o = 0; o < NOM; ++o) {
        const int j = lane + a.LS * o;
        const bool ok = o < a.NO && lane < a.LS && j < yplane;
        const int jc = ok ? j : 0;
        const int p = fdiv(jc, a.inv_q), q = jc - p * a.Q;
        xo[o] = p * ST * a.PPW + q * ST;
        yoff[o] = ok ? (unsigned)j * ESZ : kOob;   // absent pixels multiply by zero
    }

    const rsrc_t xrs = make_rsrc(a.x, a.x_bytes);
    const rsrc_t yrs = make_rsrc(a.dy, a.y_bytes);
    float acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = 0.f;

    float xv[NPI], yv[NOM];
    auto fetch = [&](int n) {
        const unsigned xb = (unsigned)((n * a.C + c) * xplane) * ESZ, yb = (unsigned)((n * a.C + c) * yplane) * ESZ;
#pragma unroll
        for (int i = 0; i < NPI; ++i) xv[i] = buf_load(xrs, xb + goff[i], tnull);
#pragma unroll
        for (int o = 0; o < NOM; ++o) yv[o] = buf_load(yrs, yb + yoff[o], tnull);
    };
    if (n0 < n1) fetch(n0);
    for (int n = n0; n < n1; ++n) {
        float yc[NOM];
#pragma unroll
        for (int i = 0; i < NPI; ++i)
            if (lane + 64 * i < PPS) my[lane + 64 * i] = xv[i];
#pragma unroll
        for (int o = 0; o < NOM; ++o) yc[o] = yv[o];
        if (n + 1 < n1) fetch(n + 1);
#pragma unroll
        for (int o = 0; o < NOM; ++o) {
            if (o >= a.NO) break;
            const float* xq = my + xo[o];
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) acc[r * 3 + s] = fmaf(yc[o], xq[r * a.PPW + s], acc[r * 3 + s]);
        }
    }
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        float v = acc[t];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        acc[t] = v;
    }
    if (lane == 0) {
        float* out = a.out + (size_t)sp * a.C * 9 + (size_t)c * 9;
#pragma unroll
        for (int t = 0; t < 9; ++t) out[t] = acc[t];
    }
}

bool is_depthwise(const Problem& pr) { return pr.groups == pr.C && pr.groups == pr.K && pr.groups > 1; }

// Planes per workgroup: fills the 256 threads' rounds of 4-output items as evenly as possible
// within an LDS budget that still lets several workgroups share a CU.
int pick_planes(int g4, int floats_per_plane, int budget_floats) {
    auto eff = [&](int pl) {
        const int items = pl * g4;
        const int rounds = (items + kThreads - 1) / kThreads;
        return (double)items / (rounds * kThreads);
    };
    double best_eff = 0.0;
    for (int pl = 1; pl <= 64 && pl * floats_per_plane <= budget_floats; ++pl)
        if (eff(pl) > best_eff) best_eff = eff(pl);
    int best = 1;
    for (int pl = 1; pl <= 64 && pl * floats_per_plane <= budget_floats; ++pl)
        if (eff(pl) >= best_eff - 0.01) best = pl;   // the largest batch among the (nearly) best
    return best;
}

constexpr int kLdsBudgetFloats = 10 * 1024;   // 40 KB per workgroup

bool stencil_args(int pass, const Problem& pr, const void* in0, const void* in1, float* out, DwArgs& a, int& stride) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw) return false;
    if (pass == 0) {
        if (pr.sh > 2) return false;
        a.src = in0; a.w = in1; a.dst = out;
        a.IH = pr.H; a.IW = pr.W; a.OH = pr.P; a.OW = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw; a.flip = 0;
        stride = pr.sh;
    } else if (pass == 1) {
        if (pr.sh != 1) return false;
        a.src = in0; a.w = in1; a.dst = out;
        a.IH = pr.P; a.IW = pr.Q; a.OH = pr.H; a.OW = pr.W; a.pad_h = pr.R - 1 - pr.ph; a.pad_w = pr.S - 1 - pr.pw;
        a.flip = 1;
        stride = 1;
    } else {
        return false;
    }
    a.planes = pr.N * pr.C; a.C = pr.C;
    a.PPH = (a.OH - 1) * stride + pr.R; a.PPW = (a.OW - 1) * stride + pr.S;
    const int pps = a.PPH * a.PPW, oplane = a.OH * a.OW;
    a.G4 = (oplane + 3) / 4;
    if (pps + 9 > kLdsBudgetFloats) return false;   // planes this large need row tiling (not built)
    a.PL = pick_planes(a.G4, pps + 9, kLdsBudgetFloats);
    a.inv_ppw = 1.0f / a.PPW; a.inv_pps = 1.0f / pps; a.inv_ow = 1.0f / a.OW; a.inv_g4 = 1.0f / a.G4;
    a.vec = (oplane % 4 == 0) && (reinterpret_cast<uintptr_t>(out) % 16 == 0);
    return true;
}

template <typename T>
hipError_t launch_stencil(const DwArgs& a, int stride, hipStream_t st) {
    const int grid = (a.planes + a.PL - 1) / a.PL;
    const size_t smem = (size_t)a.PL * (a.PPH * a.PPW + 9) * sizeof(float);
    if (stride == 1) dw_stencil_kernel<T, 3, 3, 1><<<grid, kThreads, smem, st>>>(a);
    else dw_stencil_kernel<T, 3, 3, 2><<<grid, kThreads, smem, st>>>(a);
    return hipGetLastError();
}

constexpr int kWgradIpt = 4;   // items per thread in the backward-weight kernel

bool wgrad_args(const Problem& pr, const void* x, const void* dy, DwWArgs& a) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw || pr.sh > 2) return false;
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.P = pr.P; a.Q = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.PPH = (pr.P - 1) * pr.sh + 3; a.PPW = (pr.Q - 1) * pr.sh + 3;
    const int pps = a.PPH * a.PPW, yplane = pr.P * pr.Q;
    a.G4 = (yplane + 3) / 4;
    const int per_plane = pps + yplane > a.G4 * 9 ? pps + yplane : a.G4 * 9;
    if (per_plane > kLdsBudgetFloats) return false;
    int pl = pick_planes(a.G4, per_plane, kLdsBudgetFloats);
    while (pl > 1 && pl * a.G4 > kThreads * kWgradIpt) --pl;
    if (pl * a.G4 > kThreads * kWgradIpt) return false;
    a.PL = pl;
    a.inv_ppw = 1.0f / a.PPW; a.inv_pps = 1.0f / pps; a.inv_q = 1.0f / pr.Q; a.inv_g4 = 1.0f / a.G4;
    a.cblocks = (pr.C + pl - 1) / pl;
    int nsplit = (2048 + a.cblocks - 1) / a.cblocks;   // enough workgroups in flight to cover HBM latency
    if (nsplit > pr.N) nsplit = pr.N;
    a.nsplit = nsplit;
    return true;
}

// ---- wave-private variants: host side ----------------------------------------------------------------
bool wave_shape_ok(const Problem& pr, int pps, int outs) {
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    return pps <= 1024 && outs <= 1024;
}
// Outputs per lane and lane stride: NO = ceil(outs/64), LS = ceil(outs/NO).
void lane_split(int outs, int& no, int& ls) {
    no = (outs + 63) / 64;
    ls = (outs + no - 1) / no;
}

bool wave_stencil_args(int pass, const Problem& pr, const void* in0, const void* in1, float* out, DwWaveArgs& a,
                       int& stride) {
    DwArgs b{};
    if (!stencil_args(pass, pr, in0, in1, out, b, stride)) return false;
    const int pps = b.PPH * b.PPW;
    if (!wave_shape_ok(pr, pps, b.OH * b.OW)) return false;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    a.src = b.src; a.w = b.w; a.dst = b.dst; a.planes = b.planes; a.C = b.C;
    a.IH = b.IH; a.IW = b.IW; a.OH = b.OH; a.OW = b.OW; a.pad_h = b.pad_h; a.pad_w = b.pad_w;
    a.PPH = b.PPH; a.PPW = b.PPW; a.inv_ppw = b.inv_ppw; a.inv_ow = b.inv_ow;
    lane_split(b.OH * b.OW, a.NO, a.LS);
    a.flip = b.flip;
    a.src_bytes = (unsigned)((size_t)a.planes * a.IH * a.IW * esz);
    return true;
}

template <typename T, int ST>
hipError_t launch_wave_stencil(DwWaveArgs a, hipStream_t st) {
    const int pps = a.PPH * a.PPW;
    const bool small = pps <= 256 && a.NO <= 4;
    const int pb = small ? 4 : 1;
    a.nbatches = (a.planes + pb - 1) / pb;
    int grid = (a.nbatches + 3) / 4;
    if (grid > 4096) grid = 4096;
    const size_t smem = (size_t)4 * pb * pps * sizeof(float);
    if (small) dw_wave_stencil_kernel<T, ST, 4, 4, 4><<<grid, kThreads, smem, st>>>(a);
    else dw_wave_stencil_kernel<T, ST, 16, 16, 1><<<grid, kThreads, smem, st>>>(a);
    return hipGetLastError();
}

bool wave_wgrad_args(const Problem& pr, const void* x, const void* dy, DwWaveWArgs& a) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw || pr.sh > 2) return false;
    a.PPH = (pr.P - 1) * pr.sh + 3; a.PPW = (pr.Q - 1) * pr.sh + 3;
    if (!wave_shape_ok(pr, a.PPH * a.PPW, pr.P * pr.Q)) return false;
    lane_split(pr.P * pr.Q, a.NO, a.LS);
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.P = pr.P; a.Q = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.inv_ppw = 1.0f / a.PPW; a.inv_q = 1.0f / pr.Q;
    int nsplit = (8192 + pr.C - 1) / pr.C;   // about 8192 waves in flight cover the HBM latency
    if (nsplit > pr.N) nsplit = pr.N;
    a.nsplit = nsplit;
    a.x_bytes = (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * esz);
    a.y_bytes = (unsigned)((size_t)pr.N * pr.C * pr.P * pr.Q * esz);
    return true;
}

template <typename T, int ST>
hipError_t launch_wave_wgrad(const DwWaveWArgs& a, hipStream_t st) {
    const int pps = a.PPH * a.PPW;
    const int grid = (a.C * a.nsplit + 3) / 4;
    const size_t smem = (size_t)4 * pps * sizeof(float);
    if (pps <= 256 && a.NO <= 4) dw_wave_wgrad_kernel<T, ST, 4, 4><<<grid, kThreads, smem, st>>>(a);
    else dw_wave_wgrad_kernel<T, ST, 16, 16><<<grid, kThreads, smem, st>>>(a);
    return hipGetLastError();
}

}  // namespace

bool depthwise_supports(int pass, const Problem& pr) {
    if (pass == 2) {
        DwWArgs a{};
        DwWaveWArgs b{};
        return wave_wgrad_args(pr, nullptr, nullptr, b) || wgrad_args(pr, nullptr, nullptr, a);
    }
    DwArgs a{};
    int stride;
    return stencil_args(pass, pr, nullptr, nullptr, nullptr, a, stride);
}

size_t depthwise_workspace_bytes(int pass, const Problem& pr) {
    if (pass != 2) return 0;
    DwWaveWArgs b{};
    if (wave_wgrad_args(pr, nullptr, nullptr, b)) return b.nsplit > 1 ? (size_t)b.nsplit * pr.C * 9 * sizeof(float) : 0;
    DwWArgs a{};
    if (!wgrad_args(pr, nullptr, nullptr, a)) return 0;
    return a.nsplit > 1 ? (size_t)a.nsplit * pr.C * 9 * sizeof(float) : 0;
}

hipError_t depthwise_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                         hipStream_t st) {
    const int count = pr.C * 9;
    if (pass == 2) {
        DwWaveWArgs b{};
        if (wave_wgrad_args(pr, in0, in1, b)) {
            b.out = b.nsplit > 1 ? static_cast<float*>(ws) : out;
            hipError_t e;
            if (pr.dtype == 0) e = pr.sh == 1 ? launch_wave_wgrad<float, 1>(b, st) : launch_wave_wgrad<float, 2>(b, st);
            else e = pr.sh == 1 ? launch_wave_wgrad<uint16_t, 1>(b, st) : launch_wave_wgrad<uint16_t, 2>(b, st);
            if (e != hipSuccess || b.nsplit == 1) return e;
            dw_reduce_splits_kernel<<<(count + 255) / 256, 256, 0, st>>>(static_cast<const float*>(ws), out, b.nsplit, count);
            return hipGetLastError();
        }
        DwWArgs a{};
        if (!wgrad_args(pr, in0, in1, a)) return hipErrorNotSupported;
        a.out = a.nsplit > 1 ? static_cast<float*>(ws) : out;
        const int pps = a.PPH * a.PPW, yplane = pr.P * pr.Q;
        const int per_plane = pps + yplane > a.G4 * 9 ? pps + yplane : a.G4 * 9;
        const size_t smem = (size_t)a.PL * per_plane * sizeof(float);
        const int grid = a.cblocks * a.nsplit;
        if (pr.dtype == 0) {
            if (pr.sh == 1) dw_wgrad_kernel<float, 3, 3, 1, kWgradIpt><<<grid, kThreads, smem, st>>>(a);
            else dw_wgrad_kernel<float, 3, 3, 2, kWgradIpt><<<grid, kThreads, smem, st>>>(a);
        } else {
            if (pr.sh == 1) dw_wgrad_kernel<uint16_t, 3, 3, 1, kWgradIpt><<<grid, kThreads, smem, st>>>(a);
            else dw_wgrad_kernel<uint16_t, 3, 3, 2, kWgradIpt><<<grid, kThreads, smem, st>>>(a);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || a.nsplit == 1) return e;
        dw_reduce_splits_kernel<<<(count + 255) / 256, 256, 0, st>>>(static_cast<const float*>(ws), out, a.nsplit, count);
        return hipGetLastError();
    }
    DwWaveArgs wv{};
    int stride;
    if (wave_stencil_args(pass, pr, in0, in1, out, wv, stride)) {
        if (pr.dtype == 0) return stride == 1 ? launch_wave_stencil<float, 1>(wv, st) : launch_wave_stencil<float, 2>(wv, st);
        return stride == 1 ? launch_wave_stencil<uint16_t, 1>(wv, st) : launch_wave_stencil<uint16_t, 2>(wv, st);
    }
    DwArgs a{};
    if (!stencil_args(pass, pr, in0, in1, out, a, stride)) return hipErrorNotSupported;
    return pr.dtype == 0 ? launch_stencil<float>(a, stride, st) : launch_stencil<uint16_t>(a, stride, st);
}

}  // namespace miconv
