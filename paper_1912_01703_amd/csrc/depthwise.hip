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

#include <mutex>
#include <type_traits>
#include <utility>
#include <vector>

namespace miconv {
namespace {

constexpr int kThreads = 256;

constexpr int kStream = 2;   // cache policy "non-temporal": data that is read once (3 % on the backward-weight kernel)
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

// Sums the split partials in a fixed order.  All loads of an element are issued before the first add.
__global__ __launch_bounds__(256) void dw_reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                               int nsplit, int count) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = 0.f;
    for (int s0 = 0; s0 < nsplit; s0 += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = s0 + k < nsplit ? part[(size_t)(s0 + k) * count + i] : 0.f;
#pragma unroll
        for (int k = 0; k < 8; ++k) sum += v[k];
    }
    dw[i] = sum;
}

// ====================================================================================================
// Wave-private "strip" kernels for the usual depthwise plane sizes (output width <= 64, padded plane
// <= 1024 floats: 7x7 ... 28x28, stride 1 or 2).
//
// A wave owns whole planes, so there is no workgroup barrier.  It fetches a batch of PB planes with
// coalesced row reads into its own zero-bordered LDS region while it computes the previous batch.
// In the compute step a lane owns one output column q of one 7-row segment of one plane and slides
// down it: a 9x3 window of inputs (27 LDS reads) yields 7 outputs (63 FMAs), instead of 9 reads per
// output.  Lanes of a segment read consecutive LDS words and write consecutive outputs.  Everything
// that depends only on the lane (gather offsets, window and output offsets) is computed once.
// ====================================================================================================
constexpr int kSeg = 7;   // output rows per lane

struct DwStripArgs {
    const void* src;
    const void* w;
    float* dst;
    int planes, C;
    int IH, IW, OH, OW, pad_h, pad_w;
    int PPH, PPW;
    int PB;            // planes per batch
    int NSEG;          // 7-row segments per plane
    int UPP;           // (plane, segment) units per 64-lane pass = 64 / OW
    int passes;        // ceil(PB*NSEG / UPP)
    int lds_per_wave;  // floats: [PB planes][slack rows][9*PB filter taps][PB output planes (wide path)]
    int w_off, o_off;  // where the filter taps and the output staging start inside a wave's region
    float inv_ppw, inv_pps, inv_ow, inv_nseg, inv_c, inv_iplane, inv_iw;
    int flip, nbatches;
    unsigned src_bytes, w_bytes;
    // fused epilogues of the 16-byte path (see EPI below)
    const float* bias;   // [C]
    const void* mask;    // float, shaped like dst
    unsigned dst_bytes;
};

// NPIB: 64-lane passes over the batch's padded planes (NPIB*64 >= PB*PPH*PPW).  NPS: most compute passes.
// WIDE: global memory is touched only with 16-byte accesses per lane (the texture-address unit moves a
// quarter of its peak with 4-byte ones, which is what bounds this kernel): the batch is read as
// consecutive float4 and scattered into the padded planes, results are gathered from an LDS staging
// area as float4.  Needs fp32 planes whose sizes are multiples of 4 and 16-byte aligned tensors.
// PPWC, OWC: padded-plane and output widths known at compile time (0: taken from the arguments), which
// turns every LDS offset of the compute step into an immediate.  Such an instance also assumes that the
// output height is a multiple of kSeg: every lane owns kSeg rows or none, and the per-row checks go.
// EPI (16-byte path only): 0 plain; 1 forward with bias and ReLU: the accumulator starts at the channel's bias (kept in
// LDS behind the filter taps) and is clamped at zero; 2 backward-data with a ReLU mask: the mask values under a
// batch's results are fetched together with the next batch and applied to the float4 on its way out.
template <typename T, int ST, int NPIB, int NPS, bool WIDE, int PPWC = 0, int OWC = 0, int EPI = 0>
__global__ __launch_bounds__(kThreads) void dw_strip_stencil_kernel(DwStripArgs a) {
    static_assert(EPI == 0 || (WIDE && sizeof(T) == 4), "fused epilogues exist on the 16-byte fp32 path");
    constexpr int NLV = 4;   // float4 passes over a batch's input / output (PB*plane/4 <= 256)
    extern __shared__ float lds[];
    constexpr unsigned ESZ = sizeof(T);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr bool WHOLE = PPWC != 0;
    const int ppw = PPWC ? PPWC : a.PPW, ow = OWC ? OWC : a.OW;
    const int PPS = a.PPH * ppw;
    const int iplane = a.IH * a.IW, oplane = a.OH * ow;
    const T* const tnull = nullptr;
    float* my = lds + wave * a.lds_per_wave;
    float* wl = my + a.w_off;   // behind the planes and the slack rows masked strips read
    float* ol = my + a.o_off;

    // wide path: lane's float4 f = lane + 64*i of the batch
    unsigned vgo[NLV];
    if constexpr (WIDE) {
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const int f = lane + 64 * i;
            vgo[i] = 4 * f < a.PB * iplane ? (unsigned)f * 16u : kOob;
        }
    }

    unsigned goff[NPIB];   // byte offset inside the batch, kOob = zero
#pragma unroll
    for (int i = 0; i < NPIB; ++i) {
        const int e = lane + 64 * i;
        const int pl = fdiv(e, a.inv_pps), rem = e - pl * PPS;
        const int ph = fdiv(rem, a.inv_ppw), pw = rem - ph * ppw;
        const int ih = ph - a.pad_h, iw = pw - a.pad_w;
        const bool ok = e < a.PB * PPS && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
        goff[i] = ok ? (unsigned)(pl * iplane + ih * a.IW + iw) * ESZ : kOob;
    }
    int win[NPS], oo[NPS], rows[NPS], wof[NPS], bof[NPS];
    {
        const int ul = fdiv(lane, a.inv_ow), q = lane - ul * ow;
#pragma unroll
        for (int ps = 0; ps < NPS; ++ps) {
            const int u = ps * a.UPP + ul;
            const bool ok = ps < a.passes && ul < a.UPP && u < a.PB * a.NSEG;
            const int uc = ok ? u : 0;
            const int pl = fdiv(uc, a.inv_nseg), seg = uc - pl * a.NSEG;
            const int p0 = seg * kSeg;
            win[ps] = pl * PPS + p0 * ST * ppw + q * ST;
            oo[ps] = pl * oplane + p0 * ow + q;
            rows[ps] = ok ? min(kSeg, a.OH - p0) : 0;
            wof[ps] = pl * 9;
            bof[ps] = 9 * a.PB + pl;
        }
    }

    const rsrc_t srs = make_rsrc(a.src, a.src_bytes);
    const rsrc_t wrs = make_rsrc(a.w, a.w_bytes);
    const rsrc_t mrs = make_rsrc(a.mask, EPI == 2 ? a.dst_bytes : 0u);
    const int nw = gridDim.x * (kThreads / 64);
    float v[WIDE ? 1 : NPIB];
    v4u v4[WIDE ? NLV : 1];
    v4u m4[EPI == 2 ? NLV : 1], m4cur[EPI == 2 ? NLV : 1];
    float wreg, breg = 0.f;
    // Planes past the end of the tensor lie beyond the descriptor: zeros.
    auto fetch = [&](int b) {
        const unsigned base = (unsigned)(b * a.PB * iplane) * ESZ;
        if constexpr (WIDE) {
#pragma unroll
            for (int i = 0; i < NLV; ++i) v4[i] = __builtin_amdgcn_raw_buffer_load_b128(srs, base + vgo[i], 0, 0);
        } else {
#pragma unroll
            for (int i = 0; i < NPIB; ++i) v[i] = buf_load(srs, base + goff[i], tnull);
        }
        // lane l < 9*PB fetches tap l%9 of the batch's plane l/9
        const int pl = lane / 9, t = lane - pl * 9;
        const int plane = b * a.PB + pl;
        const int c = plane - fdiv(plane, a.inv_c) * a.C;
        wreg = buf_load(wrs, (pl < a.PB && plane < a.planes) ? (unsigned)(c * 9 + (a.flip ? 8 - t : t)) * ESZ : kOob, tnull);
        if constexpr (EPI == 1) {   // lane l < PB fetches the bias of the batch's plane l
            const int bplane = b * a.PB + lane;
            const int bc = bplane - fdiv(bplane, a.inv_c) * a.C;
            breg = (lane < a.PB && bplane < a.planes) ? a.bias[bc] : 0.f;
        }
        if constexpr (EPI == 2) {   // the mask under the batch's results, as the results will be stored
            const unsigned mbase = (unsigned)(b * a.PB * oplane) * 4u;
#pragma unroll
            for (int i = 0; i < NLV; ++i) {
                const int f = lane + 64 * i;
                m4[i] = __builtin_amdgcn_raw_buffer_load_b128(mrs, 4 * f < a.PB * oplane ? mbase + (unsigned)f * 16u : kOob, 0, 0);
            }
        }
    };
    int b = blockIdx.x * (kThreads / 64) + wave;
    if (b < a.nbatches) fetch(b);   // the first batch is on its way while the rest of the plan is made

    // wide path: where the four values of float4 f land in LDS
    int lo[NLV][4];
    if constexpr (WIDE) {
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const int f = lane + 64 * i;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = 4 * f + k;
                const int pl = fdiv(idx, a.inv_iplane), rem = idx - pl * iplane;
                const int ih = fdiv(rem, a.inv_iw), iw = rem - ih * a.IW;
                const int ph = ih + a.pad_h, pw = iw + a.pad_w;
                const bool ok = idx < a.PB * iplane && ph >= 0 && ph < a.PPH && pw >= 0 && pw < ppw;
                lo[i][k] = ok ? pl * PPS + ph * ppw + pw : a.lds_per_wave - 1;   // values without a place land in a spare word
            }
        }
        // borders (and the slack) are written once; the scatter only ever touches interior words
        for (int e = lane; e < a.w_off; e += 64) my[e] = 0.f;
    }
    for (; b < a.nbatches; b += nw) {
        if constexpr (WIDE) {
#pragma unroll
            for (int i = 0; i < NLV; ++i)
#pragma unroll
                for (int k = 0; k < 4; ++k) my[lo[i][k]] = __uint_as_float(v4[i][k]);
        } else {
#pragma unroll
            for (int i = 0; i < NPIB; ++i)
                if (lane + 64 * i < a.PB * PPS) my[lane + 64 * i] = v[i];
        }
        if (lane < 9 * a.PB) wl[lane] = wreg;
        if constexpr (EPI == 1) {
            if (lane < a.PB) wl[9 * a.PB + lane] = breg;
        }
        if constexpr (EPI == 2) {
#pragma unroll
            for (int i = 0; i < NLV; ++i) m4cur[i] = m4[i];
        }
        if (b + nw < a.nbatches) fetch(b + nw);   // the next batch travels while this one is computed
        float* d = a.dst + (size_t)b * a.PB * oplane;
        const int live = min(a.PB, a.planes - b * a.PB) * oplane;   // outputs that exist in this batch
        auto pass = [&](int ps) __attribute__((always_inline)) {
            const float* xq = my + win[ps];
            float wv[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) wv[t] = wl[wof[ps] + t];
            float xw[(kSeg - 1) * ST + 3][3];
#pragma unroll
            for (int r = 0; r < (kSeg - 1) * ST + 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) xw[r][s] = xq[r * ppw + s];
            const float bias0 = EPI == 1 ? wl[bof[ps]] : 0.f;
#pragma unroll
            for (int i = 0; i < kSeg; ++i) {
                float acc = bias0;
#pragma unroll
                for (int r = 0; r < 3; ++r)
#pragma unroll
                    for (int s = 0; s < 3; ++s) acc = fmaf(xw[i * ST + r][s], wv[r * 3 + s], acc);
                if constexpr (EPI == 1) acc = fmaxf(acc, 0.f);
                const int o = oo[ps] + i * ow;
                if constexpr (WIDE) {
                    if (WHOLE || i < rows[ps]) ol[o] = acc;
                } else {
                    if ((WHOLE || i < rows[ps]) && o < live) d[o] = acc;
                }
            }
        };
#pragma unroll
        for (int ps = 0; ps < NPS; ++ps) {
            if (ps >= a.passes) break;
            if constexpr (WHOLE) {
                if (rows[ps] != 0) pass(ps);
            } else {
                pass(ps);
            }
        }
        if constexpr (WIDE) {
#pragma unroll
            for (int i = 0; i < NLV; ++i) {
                const int f = lane + 64 * i;
                // streamed past the caches: the results are not read again by this kernel, and a plain store
                // costs a fifth more time (22.2 against 18.0 us on 14x14 planes, N*C = 65 536)
                if (4 * f < live) {
                    v4f r4 = *reinterpret_cast<const v4f*>(ol + 4 * f);
                    if constexpr (EPI == 2) {
#pragma unroll
                        for (int k = 0; k < 4; ++k) r4[k] = __uint_as_float(m4cur[i][k]) > 0.f ? r4[k] : 0.f;
                    }
                    __builtin_nontemporal_store(r4, reinterpret_cast<v4f*>(d + 4 * f));
                }
            }
        }
    }
}

// Sum of v over the 64 lanes of a wave, returned to every lane, by data-parallel-primitive moves (no LDS traffic):
// four shifts inside each row of 16 lanes leave the row's total in its last lane, two broadcasts of a row's last
// lane into the following rows carry the totals to lane 63.  Lanes whose source lies outside the row (or whose row
// is masked off) receive 0.  The order of the additions is fixed.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add(float v) {
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_total(float v) {
    v = dpp_add<0x111, 0xF>(v);   // row_shr:1
    v = dpp_add<0x112, 0xF>(v);   // row_shr:2
    v = dpp_add<0x114, 0xF>(v);   // row_shr:4
    v = dpp_add<0x118, 0xF>(v);   // row_shr:8
    v = dpp_add<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v = dpp_add<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

struct DwStripWArgs {
    const void* x;
    const void* dy;
    float* out;        // [wsplit][C*9] (dw itself when wsplit == 1)
    int N, C, H, W, P, Q, pad_h, pad_w;
    int PPH, PPW;
    int PB, NSEG, UPP, passes, lds_per_wave, w_off, o_off;
    float inv_ppw, inv_pps, inv_q, inv_nseg, inv_xplane, inv_w, inv_yplane;
    int CPB, IB;       // a batch of PB planes = IB consecutive images x CPB consecutive channels
    int cgroups;       // groups of CPB consecutive channels
    int waves;         // waves per workgroup = image ranges summed inside the workgroup
    int wsplit;        // workgroups per channel group; their partial sums meet in the workspace
    unsigned x_bytes, y_bytes;
};


// One wave = CPB consecutive channels and a contiguous range of images, IB images at a time.  The CPB
// planes of an image are one contiguous run of memory, and neighbouring workgroups own neighbouring
// channels, so that the waves in flight together sweep whole images.  The nine partial sums per
// channel stay in the lanes' registers over the whole range, the next batch is fetched while the
// current one is multiplied, and at the end lanes, then the waves of the workgroup (the image
// ranges), are added in a fixed order: bit-reproducible, no atomics.
// Most waves per workgroup (two per SIMD).
constexpr int kStripWgradWaves = 8;

template <typename T, int ST, int NPIB, int NPS, bool WIDE, int PPWC = 0, int QC = 0>
__global__ __launch_bounds__(64 * kStripWgradWaves) void dw_strip_wgrad_kernel(DwStripWArgs a) {
    constexpr int NLV = 4;   // float4 passes over a batch of x / dy planes
    extern __shared__ float lds[];
    constexpr unsigned ESZ = sizeof(T);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    constexpr bool WHOLE = PPWC != 0;   // such an instance is only launched when P is a multiple of kSeg
    const int ppw = PPWC ? PPWC : a.PPW, qw = QC ? QC : a.Q;   // widths, compile-time constants where given
    const int PPS = a.PPH * ppw;
    const int xplane = a.H * a.W, yplane = a.P * qw;
    const T* const tnull = nullptr;
    float* my = lds + wave * a.lds_per_wave;
    float* wres = lds + a.waves * a.lds_per_wave;   // [wave][64]: per-wave sums
    // Consecutive workgroup ids go to different XCDs (8, one L2 each).  The channel groups are dealt out so
    // that an XCD owns a contiguous range of channels: the cache lines that two neighbouring groups share
    // (planes are not multiples of 128 bytes) are then fetched from HBM once, not once per L2.
    const int per_xcd = (a.cgroups + 7) / 8;
    const int bid = blockIdx.x % (8 * per_xcd), ws = blockIdx.x / (8 * per_xcd);
    const int cg = (bid & 7) * per_xcd + (bid >> 3);
    if ((bid >> 3) >= per_xcd || cg >= a.cgroups) return;   // the whole workgroup: no barrier is missed
    const int c0 = cg * a.CPB;
    const int parts = a.wsplit * a.waves, part = ws * a.waves + wave;
    const int nbat = (a.N + a.IB - 1) / a.IB;   // ranges are whole batches of IB images
    const int n0 = (int)((long long)nbat * part / parts) * a.IB, n1 = min(a.N, (int)((long long)nbat * (part + 1) / parts) * a.IB);
    const float inv_cpb = 1.0f / a.CPB;
    // plane pl of a batch = image pl / CPB, channel pl % CPB; its offset from (image n, channel c0) in planes
    auto plane_of = [&](int pl, int& ch) __attribute__((always_inline)) {
        const int img = fdiv(pl, inv_cpb);
        ch = pl - img * a.CPB;
        return img * a.C + ch;
    };

    float* yl = my + a.o_off;   // wide path: the batch's dy planes, unpadded

    // wide path: float4 f = lane + 64*i of the batch's x planes (and dy planes); planes are multiples of
    // 4 elements, so a float4 belongs to one plane
    unsigned vgx[NLV], vgy[NLV];
    int lo[NLV][4];   // filled once the first loads are on their way
    if constexpr (WIDE) {
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const int f = lane + 64 * i;
            const int plx = fdiv(4 * f, a.inv_xplane), ply = fdiv(4 * f, a.inv_yplane);
            int chx, chy;
            const int px = plane_of(plx, chx), py = plane_of(ply, chy);
            vgx[i] = plx < a.PB && c0 + chx < a.C ? (unsigned)(px * xplane + (4 * f - plx * xplane)) * 4u : kOob;
            vgy[i] = ply < a.PB && c0 + chy < a.C ? (unsigned)(py * yplane + (4 * f - ply * yplane)) * 4u : kOob;
        }
    }

    // offsets relative to (image n, channel c0); channels past the last one read as zeros, and so do images
    // past the wave's range (the descriptors end there)
    unsigned goff[NPIB];
#pragma unroll
    for (int i = 0; i < NPIB; ++i) {
        const int e = lane + 64 * i;
        const int pl = fdiv(e, a.inv_pps), rem = e - pl * PPS;
        const int ph = fdiv(rem, a.inv_ppw), pw = rem - ph * ppw;
        const int ih = ph - a.pad_h, iw = pw - a.pad_w;
        int ch;
        const int po = plane_of(pl, ch);
        const bool ok = e < a.PB * PPS && c0 + ch < a.C && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
        goff[i] = ok ? (unsigned)(po * xplane + ih * a.W + iw) * ESZ : kOob;
    }
    int win[NPS], rows[NPS], yli[NPS], chn[NPS];   // chn: channel (within the group) the lane works for in a pass, -1: none
    unsigned yo[NPS];
    {
        const int ul = fdiv(lane, a.inv_q), q = lane - ul * qw;
#pragma unroll
        for (int ps = 0; ps < NPS; ++ps) {
            const int u = ps * a.UPP + ul;
            const bool ok = ps < a.passes && ul < a.UPP && u < a.PB * a.NSEG;
            const int uc = ok ? u : 0;
            const int pl = fdiv(uc, a.inv_nseg), seg = uc - pl * a.NSEG;
            const int p0 = seg * kSeg;
            win[ps] = pl * PPS + p0 * ST * ppw + q * ST;
            int ch;
            const int po = plane_of(pl, ch);
            yo[ps] = c0 + ch < a.C ? (unsigned)(po * yplane + p0 * qw + q) * ESZ : kOob;
            yli[ps] = pl * yplane + p0 * qw + q;
            rows[ps] = ok ? min(kSeg, a.P - p0) : 0;
            chn[ps] = ok ? ch : -1;
        }
    }

    const int last = __builtin_amdgcn_readfirstlane((n1 - 1) * a.C + min(c0 + a.CPB, a.C));   // planes up to the range's end
    const rsrc_t xrs = make_rsrc(a.x, n1 > n0 ? (unsigned)(last * xplane) * ESZ : 0u);
    const rsrc_t yrs = make_rsrc(a.dy, n1 > n0 ? (unsigned)(last * yplane) * ESZ : 0u);
    float acc[NPS][9];
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[ps][t] = 0.f;

    // One batch in flight per wave.  With two or three register sets per wave the kernel was slower (14x14 planes,
    // N*C = 65 536: 20.3 us with one set, 21.5 with two, 24.5 with three): sixteen waves per CU with one batch each
    // already queue more requests than the memory system serves at its best rate, and the smaller register
    // footprint lets four waves share a SIMD.
    constexpr int DEPTH = 1;
    float xv[WIDE ? 1 : NPIB], yv[WIDE ? 1 : NPS][kSeg];
    v4u x4[DEPTH][WIDE ? NLV : 1], y4[DEPTH][WIDE ? NLV : 1];
    // Batches past the range lie beyond the descriptors: zeros, no traffic.
    auto fetch = [&](int n, auto setc) __attribute__((always_inline)) {
        constexpr int SET = decltype(setc)::value;
        // kOob plus a byte offset below 2^31 is still beyond the descriptor
        const unsigned xb = (unsigned)((n * a.C + c0) * xplane) * ESZ, yb = (unsigned)((n * a.C + c0) * yplane) * ESZ;
        if constexpr (WIDE) {
#pragma unroll
            for (int i = 0; i < NLV; ++i) {
                x4[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(xrs, xb + vgx[i], 0, kStream);
                y4[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(yrs, yb + vgy[i], 0, kStream);
            }
        } else {
#pragma unroll
            for (int i = 0; i < NPIB; ++i) xv[i] = buf_load(xrs, xb + goff[i], tnull);
#pragma unroll
            for (int ps = 0; ps < NPS; ++ps)
#pragma unroll
                for (int i = 0; i < kSeg; ++i)
                    yv[ps][i] = buf_load(yrs, i < rows[ps] ? yb + yo[ps] + (unsigned)(i * qw) * ESZ : kOob, tnull);
        }
    };
    auto pass = [&](int ps) __attribute__((always_inline)) {
        const float* xq = my + win[ps];
        float yc[kSeg];
#pragma unroll
        for (int i = 0; i < kSeg; ++i) yc[i] = WHOLE || i < rows[ps] ? yl[yli[ps] + i * qw] : 0.f;
        float xw[(kSeg - 1) * ST + 3][3];
#pragma unroll
        for (int r = 0; r < (kSeg - 1) * ST + 3; ++r)
#pragma unroll
            for (int s = 0; s < 3; ++s) xw[r][s] = xq[r * ppw + s];
        // rows this lane does not own are skipped outright (their window may be another plane's data)
#pragma unroll
        for (int i = 0; i < kSeg; ++i) {
            if (!WHOLE && i >= rows[ps]) continue;
#pragma unroll
            for (int r = 0; r < 3; ++r)
#pragma unroll
                for (int s = 0; s < 3; ++s) acc[ps][r * 3 + s] = fmaf(yc[i], xw[i * ST + r][s], acc[ps][r * 3 + s]);
        }
    };
    // One batch: registers -> LDS, refill the registers with the batch DEPTH ahead, multiply.
    auto step = [&](int n, auto setc) __attribute__((always_inline)) {
        constexpr int SET = decltype(setc)::value;
        if constexpr (WIDE) {
#pragma unroll
            for (int i = 0; i < NLV; ++i) {
#pragma unroll
                for (int k = 0; k < 4; ++k) my[lo[i][k]] = __uint_as_float(x4[SET][i][k]);
                const int f = lane + 64 * i;
                if (4 * f < a.PB * yplane)
                    *reinterpret_cast<float4*>(yl + 4 * f) =
                        make_float4(__uint_as_float(y4[SET][i].x), __uint_as_float(y4[SET][i].y), __uint_as_float(y4[SET][i].z),
                                    __uint_as_float(y4[SET][i].w));
            }
        } else {
#pragma unroll
            for (int i = 0; i < NPIB; ++i)
                if (lane + 64 * i < a.PB * PPS) my[lane + 64 * i] = xv[i];
#pragma unroll
            for (int ps = 0; ps < NPS; ++ps)
#pragma unroll
                for (int i = 0; i < kSeg; ++i)
                    if (i < rows[ps]) yl[yli[ps] + i * qw] = yv[ps][i];   // dy goes through LDS too: the registers are refilled next
        }
        fetch(n + DEPTH * a.IB, setc);
#pragma unroll
        for (int ps = 0; ps < NPS; ++ps) {
            if (ps >= a.passes) break;
            if constexpr (WHOLE) {
                if (rows[ps] != 0) pass(ps);
            } else {
                pass(ps);
            }
        }
    };
    fetch(n0, std::integral_constant<int, 0>{});   // on their way while the rest of the plan is made

    // wide path: where the four values of float4 f of the x planes land in LDS
    if constexpr (WIDE) {
#pragma unroll
        for (int i = 0; i < NLV; ++i) {
            const int f = lane + 64 * i;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int idx = 4 * f + k;
                const int pl = fdiv(idx, a.inv_xplane), rem = idx - pl * xplane;
                const int ih = fdiv(rem, a.inv_w), iw = rem - ih * a.W;
                const int ph = ih + a.pad_h, pw = iw + a.pad_w;
                const bool ok = idx < a.PB * xplane && ph >= 0 && ph < a.PPH && pw >= 0 && pw < ppw;
                lo[i][k] = ok ? pl * PPS + ph * ppw + pw : a.lds_per_wave - 1;   // values without a place land in a spare word
            }
        }
        for (int e = lane; e < a.w_off; e += 64) my[e] = 0.f;   // borders and slack, written once
    }
    for (int n = n0; n < n1; n += DEPTH * a.IB) {
        step(n, std::integral_constant<int, 0>{});
    }

    // Lanes -> channels, without a trip through LDS: for every channel of the group, the sums of the lanes (and
    // passes) that worked for it are added over the wave in registers, in a fixed order.  (Through LDS, with the
    // 9 * CPB receiving lanes walking their share one read after the other, this took 2 us of 23 on 14x14 planes.)
    const int opl = lane / 9, ot = lane - opl * 9;
    float sum = 0.f;
    for (int ch = 0; ch < a.CPB; ++ch) {
        float v[9];
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            v[t] = 0.f;
#pragma unroll
            for (int ps = 0; ps < NPS; ++ps) v[t] += chn[ps] == ch ? acc[ps][t] : 0.f;
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const float tot = wave_total(v[t]);
            sum = (opl == ch && ot == t) ? tot : sum;
        }
    }
    wres[wave * 64 + lane] = sum;
    // Image ranges -> total, in range order.
    __syncthreads();
    if (wave == 0 && opl < a.CPB && c0 + opl < a.C) {
        float total = wres[lane];
        for (int w2 = 1; w2 < a.waves; ++w2) total += wres[w2 * 64 + lane];
        a.out[(size_t)ws * a.C * 9 + (size_t)(c0 + opl) * 9 + ot] = total;
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

// ---- strip kernels: host side ----------------------------------------------------------------------------
struct StripPlan {
    int PB, NSEG, UPP, passes, lds_per_wave, w_off, o_off;
};

// false when the plane shape does not fit the strip kernels (then the workgroup-level kernels run).
bool strip_plan(const Problem& pr, int oh, int ow, int pph, int ppw, int stride, int iplane, StripPlan& sp) {
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    // The strip kernels derive a plane's channel with a single-precision reciprocal, which is exact only for
    // plane numbers well below 2^23.
    if ((long long)pr.N * pr.C >= (1ll << 22)) return false;
    const int pps = pph * ppw;
    if (pr.dtype == 0 && ow < 8) return false;   // rows this short: the row kernels are a little faster (7x7: 18.4 -> 16.6 us)
    if (ow > 64 || pps > 1024) return false;
    sp.NSEG = (oh + kSeg - 1) / kSeg;
    sp.UPP = 64 / ow;
    int pb = 0;
    for (int cand = 1; cand <= 28 && cand * pps <= 1024 && cand * 9 <= 64 && cand * iplane <= 1024 &&
                       cand * oh * ow <= 1024; ++cand)
        if ((cand * sp.NSEG + sp.UPP - 1) / sp.UPP <= 2) pb = cand;
    if (pb == 0) return false;
    sp.PB = pb;
    sp.passes = (pb * sp.NSEG + sp.UPP - 1) / sp.UPP;
    sp.w_off = (pb * pps + (kSeg * stride + 3) * ppw + 3) & ~3;
    sp.o_off = (sp.w_off + 10 * pb + 3) & ~3;   // nine taps and one bias per plane
    sp.lds_per_wave = ((sp.o_off + pb * oh * ow + 3) & ~3) + 4;   // the last word takes values that have no place
    return true;
}

bool strip_stencil_args(int pass, const Problem& pr, const void* in0, const void* in1, float* out, DwStripArgs& a,
                        int& stride) {
    DwArgs b{};
    if (!stencil_args(pass, pr, in0, in1, out, b, stride)) return false;
    StripPlan sp;
    if (!strip_plan(pr, b.OH, b.OW, b.PPH, b.PPW, stride, b.IH * b.IW, sp)) return false;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    a.src = b.src; a.w = b.w; a.dst = b.dst; a.planes = b.planes; a.C = b.C;
    a.IH = b.IH; a.IW = b.IW; a.OH = b.OH; a.OW = b.OW; a.pad_h = b.pad_h; a.pad_w = b.pad_w;
    a.PPH = b.PPH; a.PPW = b.PPW;
    a.PB = sp.PB; a.NSEG = sp.NSEG; a.UPP = sp.UPP; a.passes = sp.passes; a.lds_per_wave = sp.lds_per_wave;
    a.w_off = sp.w_off; a.o_off = sp.o_off;
    a.inv_ppw = b.inv_ppw; a.inv_pps = b.inv_pps; a.inv_ow = b.inv_ow;
    a.inv_nseg = 1.0f / sp.NSEG; a.inv_c = 1.0f / pr.C; a.inv_iplane = 1.0f / (b.IH * b.IW); a.inv_iw = 1.0f / b.IW;
    a.flip = b.flip;
    a.nbatches = (a.planes + sp.PB - 1) / sp.PB;
    a.src_bytes = (unsigned)((size_t)a.planes * a.IH * a.IW * esz);
    a.w_bytes = (unsigned)((size_t)pr.C * 9 * esz);
    return true;
}

// *fused is set when the launched instance applies the problem's epilogue (bias + ReLU or ReLU mask) itself.
template <typename T, int ST>
hipError_t launch_strip_stencil(const DwStripArgs& a, hipStream_t st, bool* fused) {
    // Persistent waves: each keeps one batch in flight while it computes the previous one.
    // The grid is what is resident at once (256 CUs x the occupancy the register budget allows).
    const size_t smem = (size_t)4 * a.lds_per_wave * sizeof(float);
    const bool wide = sizeof(T) == 4 && (a.IH * a.IW) % 4 == 0 && (a.OH * a.OW) % 4 == 0 &&
                      reinterpret_cast<uintptr_t>(a.src) % 16 == 0 && reinterpret_cast<uintptr_t>(a.dst) % 16 == 0;
    // Workgroups per CU: registers allow 4 for the 16-byte stride-1 kernel (3 otherwise), LDS 160 KB.
    int occ = wide && ST == 1 ? 4 : 3;
    if (sizeof(T) == 4 && wide && a.mask) occ = ST == 1 ? 3 : 2;   // the mask instance holds a second set of float4 registers
    while (occ > 1 && occ * smem > 160 * 1024) --occ;
    const int resident = 256 * occ;
    // Every wave runs the same number of batches (a grid of `resident` would leave most waves idle in
    // the last of ceil(5.33) rounds on a 16 384-batch layer).
    const int wg_batches = (a.nbatches + 3) / 4;
    const int rounds = (wg_batches + resident - 1) / resident;
    const int grid = (wg_batches + rounds - 1) / rounds;
    const bool fixed = wide && ST == 1 && a.PPW == 16 && a.OW == 14 && a.OH % kSeg == 0;   // 14x14 planes, padding 1
    if constexpr (sizeof(T) == 4) {
        const bool mask_ok = a.mask && reinterpret_cast<uintptr_t>(a.mask) % 16 == 0;
        if (wide && (a.bias || mask_ok)) {
            *fused = true;
            if (a.bias) {
                if (fixed) dw_strip_stencil_kernel<T, 1, 16, 2, true, 16, 14, 1><<<grid, kThreads, smem, st>>>(a);
                else dw_strip_stencil_kernel<T, ST, 16, 2, true, 0, 0, 1><<<grid, kThreads, smem, st>>>(a);
            } else {
                if (fixed) dw_strip_stencil_kernel<T, 1, 16, 2, true, 16, 14, 2><<<grid, kThreads, smem, st>>>(a);
                else dw_strip_stencil_kernel<T, ST, 16, 2, true, 0, 0, 2><<<grid, kThreads, smem, st>>>(a);
            }
            return hipGetLastError();
        }
    }
    if (fixed) dw_strip_stencil_kernel<T, 1, 16, 2, true, 16, 14><<<grid, kThreads, smem, st>>>(a);
    else if (wide) dw_strip_stencil_kernel<T, ST, 16, 2, true><<<grid, kThreads, smem, st>>>(a);
    else dw_strip_stencil_kernel<T, ST, 16, 2, false><<<grid, kThreads, smem, st>>>(a);
    return hipGetLastError();
}

// One wave per (channel group, image range), about two waves per SIMD in total (256 CUs x 4 SIMDs x 2),
// each running a prefetched image loop.  Up to wmax ranges are the waves of one workgroup; beyond that
// several workgroups share a channel group and a second kernel adds their partial sums.
void split_images(DwStripWArgs& a, int wmax) {
    while (wmax > 1 && (size_t)wmax * (a.lds_per_wave + 64) * sizeof(float) > 160 * 1024) wmax /= 2;   // LDS of one CU
    const int nbat = (a.N + a.IB - 1) / a.IB;
    int parts = (2048 + a.cgroups - 1) / a.cgroups;
    if (parts > nbat) parts = nbat;
    if (parts < 1) parts = 1;
    if (parts <= wmax) {
        a.waves = parts;
        a.wsplit = 1;
    } else {
        a.waves = wmax;
        a.wsplit = (parts + wmax - 1) / wmax;
        if (a.wsplit * wmax > nbat) a.wsplit = nbat / wmax;
    }
}

bool strip_wgrad_args(const Problem& pr, const void* x, const void* dy, DwStripWArgs& a) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw || pr.sh > 2) return false;
    a.PPH = (pr.P - 1) * pr.sh + 3; a.PPW = (pr.Q - 1) * pr.sh + 3;
    StripPlan sp;
    if (!strip_plan(pr, pr.P, pr.Q, a.PPH, a.PPW, pr.sh, pr.H * pr.W, sp)) return false;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.P = pr.P; a.Q = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.PB = sp.PB; a.NSEG = sp.NSEG; a.UPP = sp.UPP; a.passes = sp.passes; a.lds_per_wave = sp.lds_per_wave;
    a.w_off = sp.w_off; a.o_off = sp.o_off;
    a.inv_ppw = 1.0f / a.PPW; a.inv_pps = 1.0f / (a.PPH * a.PPW); a.inv_q = 1.0f / pr.Q; a.inv_nseg = 1.0f / sp.NSEG;
    a.inv_xplane = 1.0f / (pr.H * pr.W); a.inv_w = 1.0f / pr.W; a.inv_yplane = 1.0f / (pr.P * pr.Q);
    if (a.lds_per_wave < 2 * 64 * 9) a.lds_per_wave = 2 * 64 * 9;   // the lane sums of both passes
    // As many consecutive channels per wave as still leave two workgroups for every CU (they run at different
    // points of their image ranges, so one's start-up and final reduction overlap the other's loads: 20.3 -> 19.9 us
    // on 14x14 planes, N*C = 65 536); the rest of the batch are further images of the same channels.
    a.CPB = 1;
    for (int d = 2; d <= sp.PB; ++d)
        if (sp.PB % d == 0 && (pr.C + d - 1) / d >= 512) a.CPB = d;
    a.IB = sp.PB / a.CPB;
    a.cgroups = (pr.C + a.CPB - 1) / a.CPB;
    split_images(a, kStripWgradWaves);
    a.x_bytes = (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * esz);
    a.y_bytes = (unsigned)((size_t)pr.N * pr.C * pr.P * pr.Q * esz);
    return true;
}

// Allows a kernel the whole 160 KB of a CU as dynamic LDS; asked of the runtime once per (device, kernel).
hipError_t grant_lds(const void* kernel) {
    static std::mutex mu;
    static std::vector<std::pair<int, const void*>> granted;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    for (const auto& g : granted)
        if (g.first == dev && g.second == kernel) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) granted.emplace_back(dev, kernel);
    return e;
}

// Launches the kernel; *wsplit tells the caller how many partial sums per element it left in a.out.
template <typename T, int ST>
hipError_t launch_strip_wgrad(DwStripWArgs a, float* dw, int* wsplit, hipStream_t st) {
    const bool wide = sizeof(T) == 4 && (a.H * a.W) % 4 == 0 && (a.P * a.Q) % 4 == 0 &&
                      reinterpret_cast<uintptr_t>(a.x) % 16 == 0 && reinterpret_cast<uintptr_t>(a.dy) % 16 == 0;
    const bool fixed = wide && ST == 1 && a.PPW == 16 && a.Q == 14 && a.P % kSeg == 0;   // 14x14 planes, padding 1
    split_images(a, kStripWgradWaves);
    if (a.wsplit == 1) a.out = dw;
    *wsplit = a.wsplit;
    const int grid = 8 * ((a.cgroups + 7) / 8) * a.wsplit;
    const size_t smem = ((size_t)a.waves * a.lds_per_wave + (size_t)a.waves * 64) * sizeof(float);
    auto kernel = wide ? dw_strip_wgrad_kernel<T, ST, 16, 2, true> : dw_strip_wgrad_kernel<T, ST, 16, 2, false>;
    if constexpr (ST == 1) {
        if (fixed) kernel = dw_strip_wgrad_kernel<T, 1, 16, 2, true, 16, 14>;
    }
    if (smem > 64 * 1024) {   // dynamic LDS beyond 64 KB has to be granted first
        const hipError_t e = grant_lds(reinterpret_cast<const void*>(kernel));
        if (e != hipSuccess) return e;
    }
    kernel<<<grid, 64 * a.waves, smem, st>>>(a);
    return hipGetLastError();
}

// ====================================================================================================
// Row kernels: planes of any size, no LDS.  A thread produces four neighbouring outputs of one row
// (one 16-byte store) from bounds-checked 4-byte buffer loads; a workgroup covers consecutive rows
// of a plane, so the rows its threads share come out of the L1/L2 caches.  Used where a
// padded plane does not fit the strip kernels' LDS regions (112x112, 56x56 planes) and for
// backward-data at stride 2, which the LDS kernels do not do.
// ====================================================================================================
// n / d for n < 2^31 through a double-precision reciprocal (the integer divide of the compiler takes some forty
// instructions, and 64-bit ones far more, which bounded the row kernels: they run one short thread per four outputs).
__device__ __forceinline__ unsigned udiv(unsigned n, unsigned d, double inv) {
    unsigned q = (unsigned)((double)n * inv);
    const int r = (int)(n - q * d);
    if (r < 0) --q;
    else if ((unsigned)r >= d) ++q;
    return q;
}

// NC consecutive floats of a row starting at byte offset `off` (kOob: none), as 16-, 8- and 4-byte loads.  They need no
// more than 4-byte alignment, and words past the end of the tensor read as zero one by one.  Columns left or right of
// the row (iw0 + j outside [0, IW)) hold the neighbouring rows' values and are cleared.
template <int NC>
__device__ __forceinline__ void load_window(rsrc_t srs, unsigned off, int iw0, int IW, float (&xv)[NC]) {
#pragma unroll
    for (int j0 = 0; j0 < NC; j0 += 4) {
        if (NC - j0 >= 4) {
            const v4u v = __builtin_amdgcn_raw_buffer_load_b128(srs, off + 4u * j0, 0, 0);
#pragma unroll
            for (int k = 0; k < 4; ++k) xv[j0 + k] = __uint_as_float(v[k]);
        } else if (NC - j0 >= 2) {
            const v2u v = __builtin_amdgcn_raw_buffer_load_b64(srs, off + 4u * j0, 0, 0);
            xv[j0] = __uint_as_float(v[0]); xv[j0 + 1] = __uint_as_float(v[1]);
            if (NC - j0 == 3) xv[j0 + 2] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(srs, off + 4u * (j0 + 2), 0, 0));
        } else {
            xv[j0] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(srs, off + 4u * j0, 0, 0));
        }
    }
#pragma unroll
    for (int j = 0; j < NC; ++j)
        if (iw0 + j < 0 || iw0 + j >= IW) xv[j] = 0.f;
}

struct DwRowArgs {
    const void* src;   // x (forward) or dy (backward-data)
    const void* w;
    float* dst;
    int planes, C;
    int IH, IW, OH, OW;    // source and destination plane sizes
    int pad_h, pad_w;
    int flip;              // stride-1 backward-data = forward with the filter rotated by 180 degrees
    int bx;                // groups of four columns per row
    double inv_bx, inv_oh; // reciprocals for the item decoding
    long long items;       // planes * OH * bx
    unsigned src_bytes, w_bytes;
};

// BWD2: backward-data of a stride-2 convolution, dst = dx, src = dy:
//   dx[h][w] = sum over taps (r, s) with (h + pad - r) and (w + pad - s) even of dy[(h+pad-r)/2][(w+pad-s)/2] w[r][s];
// otherwise dst[oh][ow] = sum_{r,s} src[oh*ST - pad + r][ow*ST - pad + s] w[r][s].
template <typename T, int ST, bool BWD2>
__global__ __launch_bounds__(256) void dw_rows_kernel(DwRowArgs a) {
    constexpr unsigned ESZ = sizeof(T);
    const T* const tnull = nullptr;
    // items (plane, row, group of four columns) in row-major order, 256 per workgroup: small planes share a
    // workgroup, large ones give it a band of rows
    const long long item = (long long)blockIdx.x * 256 + threadIdx.x;
    if (item >= a.items) return;
    int qi, oh, plane;
    if (a.items < (1ll << 31)) {   // the usual case: 32-bit quotients through a double-precision reciprocal
        const unsigned rest = udiv((unsigned)item, (unsigned)a.bx, a.inv_bx);
        qi = (int)((unsigned)item - rest * (unsigned)a.bx);
        plane = (int)udiv(rest, (unsigned)a.OH, a.inv_oh);
        oh = (int)(rest - (unsigned)plane * (unsigned)a.OH);
    } else {
        qi = (int)(item % a.bx);
        const long long rest = item / a.bx;
        oh = (int)(rest % a.OH); plane = (int)(rest / a.OH);
    }
    const int ow0 = qi * 4;
    const int c = plane % a.C;
    const rsrc_t srs = make_rsrc(a.src, a.src_bytes), wrs = make_rsrc(a.w, a.w_bytes);
    float wv[9];
    if (sizeof(T) == 4) {   // the channel's nine weights as 16 + 16 + 4 bytes
        float wr[9];
        load_window<9>(wrs, (unsigned)(c * 9) * 4u, 0, 9, wr);
#pragma unroll
        for (int t = 0; t < 9; ++t) wv[t] = a.flip ? wr[8 - t] : wr[t];
    } else {
#pragma unroll
        for (int t = 0; t < 9; ++t) wv[t] = buf_load(wrs, (unsigned)(c * 9 + (a.flip ? 8 - t : t)) * ESZ, tnull);
    }
    const unsigned pbase = (unsigned)plane * (unsigned)(a.IH * a.IW);
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    if constexpr (!BWD2) {
        constexpr int NC = 3 * ST + 3;   // source columns under four outputs
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int ih = oh * ST - a.pad_h + r;
            const bool rok = ih >= 0 && ih < a.IH;
            float xv[NC];
            const int iw0 = ow0 * ST - a.pad_w;
            const long long first = (long long)pbase + (long long)ih * a.IW + iw0;   // element index of the window's first column
            if (sizeof(T) == 4 && first >= 0) {
                load_window<NC>(srs, rok ? (unsigned)first * 4u : kOob, iw0, a.IW, xv);
            } else {
#pragma unroll
                for (int j = 0; j < NC; ++j) {
                    const int iw = iw0 + j;
                    xv[j] = buf_load(srs, rok && iw >= 0 && iw < a.IW ? (pbase + (unsigned)(ih * a.IW + iw)) * ESZ : kOob, tnull);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int ss = 0; ss < 3; ++ss) acc[i] = fmaf(xv[i * ST + ss], wv[r * 3 + ss], acc[i]);
        }
    } else if (sizeof(T) == 4 && (plane > 0 || ow0 + a.pad_w >= 2)) {   // (the window may start one column left of the row: not before the tensor)
        // Column u = ow0 + i + pad_w - s of the stride-1 grid holds dy column u / 2 when u is even.  With
        // ow0 + pad_w = 2 m + e the four outputs need dy columns m - 1 .. m + 2 at most: one 16-byte load per
        // contributing row, element (e + i - s) / 2 + 1 of it for output i and tap s.
        const int e = (ow0 + a.pad_w) & 1, m = (ow0 + a.pad_w) >> 1;
        auto rows3 = [&](auto ec) __attribute__((always_inline)) {
            constexpr int E = decltype(ec)::value;
#pragma unroll
            for (int r = 0; r < 3; ++r) {
                const int t = oh + a.pad_h - r;
                const bool rok = t >= 0 && (t & 1) == 0 && (t >> 1) < a.IH;
                float yv[4];
                load_window<4>(srs, rok ? (pbase + (unsigned)((t >> 1) * a.IW + m - 1)) * 4u : kOob, m - 1, a.IW, yv);
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int ss = 0; ss < 3; ++ss)
                        if ((E + i - ss) % 2 == 0) acc[i] = fmaf(yv[(E + i - ss) / 2 + 1], wv[r * 3 + ss], acc[i]);
            }
        };
        if (e == 0) rows3(std::integral_constant<int, 0>{});
        else rows3(std::integral_constant<int, 1>{});
    } else {
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int t = oh + a.pad_h - r;
            const bool rok = t >= 0 && (t & 1) == 0 && (t >> 1) < a.IH;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int ss = 0; ss < 3; ++ss) {
                    const int u = ow0 + i + a.pad_w - ss;
                    const bool ok = rok && u >= 0 && (u & 1) == 0 && (u >> 1) < a.IW;
                    const float v = buf_load(srs, ok ? (pbase + (unsigned)((t >> 1) * a.IW + (u >> 1))) * ESZ : kOob, tnull);
                    acc[i] = fmaf(v, wv[r * 3 + ss], acc[i]);
                }
        }
    }
    float* o = a.dst + (size_t)plane * a.OH * a.OW + (size_t)oh * a.OW + ow0;
    if (ow0 + 4 <= a.OW && reinterpret_cast<uintptr_t>(o) % 16 == 0) {
        __builtin_nontemporal_store(v4f{acc[0], acc[1], acc[2], acc[3]}, reinterpret_cast<v4f*>(o));   // streamed past the caches
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (ow0 + i < a.OW) o[i] = acc[i];
    }
}

// false when the shape is not a 3x3 depthwise forward / backward-data this kernel family does.
bool rows_args(int pass, const Problem& pr, const void* in0, const void* in1, float* out, DwRowArgs& a, int& st, bool& bwd2) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw || pr.sh > 2 || pass > 1) return false;
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    a.src = in0; a.w = in1; a.dst = out;
    a.planes = pr.N * pr.C; a.C = pr.C;
    bwd2 = pass == 1 && pr.sh == 2;
    if (pass == 0) {
        a.IH = pr.H; a.IW = pr.W; a.OH = pr.P; a.OW = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw; a.flip = 0;
        st = pr.sh;
    } else {
        a.IH = pr.P; a.IW = pr.Q; a.OH = pr.H; a.OW = pr.W;
        a.pad_h = bwd2 ? pr.ph : 2 - pr.ph; a.pad_w = bwd2 ? pr.pw : 2 - pr.pw;
        a.flip = bwd2 ? 0 : 1;
        st = bwd2 ? 2 : 1;
    }
    a.bx = (a.OW + 3) / 4;
    a.inv_bx = 1.0 / a.bx; a.inv_oh = 1.0 / a.OH;
    a.items = (long long)a.planes * a.OH * a.bx;
    if ((a.items + 255) / 256 >= (1ll << 31)) return false;
    a.src_bytes = (unsigned)((size_t)a.planes * a.IH * a.IW * esz);
    a.w_bytes = (unsigned)((size_t)pr.C * 9 * esz);
    return true;
}

template <typename T>
hipError_t launch_rows(const DwRowArgs& a, int st, bool bwd2, hipStream_t stream) {
    const unsigned grid = (unsigned)((a.items + 255) / 256);
    if (bwd2) dw_rows_kernel<T, 2, true><<<grid, 256, 0, stream>>>(a);
    else if (st == 1) dw_rows_kernel<T, 1, false><<<grid, 256, 0, stream>>>(a);
    else dw_rows_kernel<T, 2, false><<<grid, 256, 0, stream>>>(a);
    return hipGetLastError();
}

// Backward-weight without LDS staging, for planes of any size.  A workgroup owns one channel and a contiguous
// share of its (image, output row, group of four columns) items; a thread adds 4 x 9 products per item into
// nine sums, which are then combined over the workgroup in a fixed order (lanes by butterfly, waves in order).
// Partial sums of the workgroups of a channel go to the workspace and are added by a second kernel.
struct DwRowWArgs {
    const void* x;
    const void* dy;
    float* out;            // [nsplit][C*9], or dw when nsplit == 1
    int N, C, H, W, P, Q, pad_h, pad_w;
    int qd;                // groups of four output columns per row
    double inv_qd, inv_p;  // reciprocals for the item decoding
    int nsplit;
    long long items;       // N * P * qd
    unsigned x_bytes, y_bytes;
};

template <typename T, int ST>
__global__ __launch_bounds__(256) void dw_rows_wgrad_kernel(DwRowWArgs a) {
    constexpr unsigned ESZ = sizeof(T);
    constexpr int NC = 3 * ST + 3;
    __shared__ float red[4 * 9];
    const T* const tnull = nullptr;
    const int c = blockIdx.x % a.C, sp = blockIdx.x / a.C;
    const long long e0 = a.items * sp / a.nsplit, e1 = a.items * (sp + 1) / a.nsplit;
    const rsrc_t xrs = make_rsrc(a.x, a.x_bytes), yrs = make_rsrc(a.dy, a.y_bytes);
    float acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = 0.f;
    for (long long e = e0 + threadIdx.x; e < e1; e += 256) {
        int q0, p, n;
        if (a.items < (1ll << 31)) {
            const unsigned rest = udiv((unsigned)e, (unsigned)a.qd, a.inv_qd);
            q0 = (int)((unsigned)e - rest * (unsigned)a.qd) * 4;
            n = (int)udiv(rest, (unsigned)a.P, a.inv_p);
            p = (int)(rest - (unsigned)n * (unsigned)a.P);
        } else {
            q0 = (int)(e % a.qd) * 4;
            const long long rest = e / a.qd;
            p = (int)(rest % a.P); n = (int)(rest / a.P);
        }
        const unsigned ybase = (unsigned)(((n * a.C + c) * a.P + p) * a.Q);
        float yv[4];
        if (sizeof(T) == 4) {
            load_window<4>(yrs, (ybase + (unsigned)q0) * 4u, q0, a.Q, yv);
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) yv[i] = buf_load(yrs, q0 + i < a.Q ? (ybase + (unsigned)(q0 + i)) * ESZ : kOob, tnull);
        }
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int ih = p * ST - a.pad_h + r;
            const bool rok = ih >= 0 && ih < a.H;
            const int iw0 = q0 * ST - a.pad_w;
            const long long first = ((long long)(n * a.C + c) * a.H + ih) * a.W + iw0;
            float xv[NC];
            if (sizeof(T) == 4 && first >= 0) {
                load_window<NC>(xrs, rok ? (unsigned)first * 4u : kOob, iw0, a.W, xv);
            } else {
                const unsigned xbase = (unsigned)(((n * a.C + c) * a.H + ih) * a.W);
#pragma unroll
                for (int j = 0; j < NC; ++j) {
                    const int iw = iw0 + j;
                    xv[j] = buf_load(xrs, rok && iw >= 0 && iw < a.W ? (xbase + (unsigned)iw) * ESZ : kOob, tnull);
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int ss = 0; ss < 3; ++ss) acc[r * 3 + ss] = fmaf(yv[i], xv[i * ST + ss], acc[r * 3 + ss]);
        }
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        float v = acc[t];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
        if (lane == 0) red[wave * 9 + t] = v;
    }
    __syncthreads();
    if (threadIdx.x < 9) {
        const float sum = ((red[threadIdx.x] + red[9 + threadIdx.x]) + red[18 + threadIdx.x]) + red[27 + threadIdx.x];
        a.out[(size_t)sp * a.C * 9 + (size_t)c * 9 + threadIdx.x] = sum;
    }
}

bool rows_wgrad_args(const Problem& pr, const void* x, const void* dy, DwRowWArgs& a) {
    if (!is_depthwise(pr) || pr.R != 3 || pr.S != 3 || pr.sh != pr.sw || pr.sh > 2) return false;
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.P = pr.P; a.Q = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.qd = (pr.Q + 3) / 4;
    a.inv_qd = 1.0 / a.qd; a.inv_p = 1.0 / pr.P;
    a.items = (long long)pr.N * pr.P * a.qd;
    // about 4096 workgroups, each with at least four items per thread
    long long ns = (4096 + pr.C - 1) / pr.C;
    const long long most = a.items / 1024 > 0 ? a.items / 1024 : 1;
    if (ns > most) ns = most;
    a.nsplit = (int)ns;
    a.x_bytes = (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * esz);
    a.y_bytes = (unsigned)((size_t)pr.N * pr.C * pr.P * pr.Q * esz);
    return true;
}


// Which kernel family serves a pass.  depthwise_supports, depthwise_workspace_bytes and depthwise_run all ask
// these two functions, so a problem that is accepted always has a kernel to run on.
enum class WPath { none, strip, rows, lds };
enum class SPath { none, strip, lds, rows };

WPath wgrad_path(const Problem& pr) {
    DwStripWArgs b{};
    if (strip_wgrad_args(pr, nullptr, nullptr, b)) return WPath::strip;
    DwWArgs a{};
    DwRowWArgs r{};
    const bool lds = wgrad_args(pr, nullptr, nullptr, a), rows = rows_wgrad_args(pr, nullptr, nullptr, r);
    // fp32: the row kernel (16-byte loads) beats the LDS kernel; bf16: the other way round
    if (pr.dtype == 0) return rows ? WPath::rows : lds ? WPath::lds : WPath::none;
    return lds ? WPath::lds : rows ? WPath::rows : WPath::none;
}

SPath stencil_path(int pass, const Problem& pr) {
    int stride;
    bool bwd2;
    DwStripArgs sa{};
    if (strip_stencil_args(pass, pr, nullptr, nullptr, nullptr, sa, stride)) return SPath::strip;
    DwArgs a{};
    DwRowArgs ra{};
    const bool lds = stencil_args(pass, pr, nullptr, nullptr, nullptr, a, stride);
    const bool rows = rows_args(pass, pr, nullptr, nullptr, nullptr, ra, stride, bwd2);
    // bf16 planes that fit the LDS budget of a workgroup: the row kernel reads bf16 two bytes at a time
    if (pr.dtype != 0 && lds) return SPath::lds;
    // larger planes, and backward-data at stride 2: the row kernels
    return rows ? SPath::rows : lds ? SPath::lds : SPath::none;
}

}  // namespace

bool depthwise_supports(int pass, const Problem& pr) {
    return pass == 2 ? wgrad_path(pr) != WPath::none : stencil_path(pass, pr) != SPath::none;
}

const char* depthwise_path_name(int pass, const Problem& pr) {
    if (pass == 2) {
        switch (wgrad_path(pr)) {
            case WPath::strip: return "depthwise/strip";
            case WPath::rows: return "depthwise/rows";
            case WPath::lds: return "depthwise/lds";
            default: return "none";
        }
    }
    switch (stencil_path(pass, pr)) {
        case SPath::strip: return "depthwise/strip";
        case SPath::rows: return "depthwise/rows";
        case SPath::lds: return "depthwise/lds";
        default: return "none";
    }
}

size_t depthwise_workspace_bytes(int pass, const Problem& pr) {
    if (pass != 2) return 0;
    int nsplit = 1;
    switch (wgrad_path(pr)) {
        case WPath::strip: { DwStripWArgs b{}; strip_wgrad_args(pr, nullptr, nullptr, b); nsplit = b.wsplit; break; }
        case WPath::lds: { DwWArgs a{}; wgrad_args(pr, nullptr, nullptr, a); nsplit = a.nsplit; break; }
        case WPath::rows: { DwRowWArgs r{}; rows_wgrad_args(pr, nullptr, nullptr, r); nsplit = r.nsplit; break; }
        default: return 0;
    }
    return nsplit > 1 ? (size_t)nsplit * pr.C * 9 * sizeof(float) : 0;
}

bool depthwise_fuses_epilogue(int pass, const Problem& pr) {
    // (given 16-byte aligned tensors; depthwise_run reports what the launch really did)
    return pass < 2 && pr.dtype == 0 && stencil_path(pass, pr) == SPath::strip && (pr.H * pr.W) % 4 == 0 && (pr.P * pr.Q) % 4 == 0;
}

hipError_t depthwise_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                         hipStream_t st, bool* fused) {
    *fused = false;
    const int count = pr.C * 9;
    if (pass == 2) {
        const WPath path = wgrad_path(pr);
        if (path == WPath::none) return hipErrorNotSupported;
        DwStripWArgs b{};
        if (path == WPath::strip) {
            strip_wgrad_args(pr, in0, in1, b);
            b.out = static_cast<float*>(ws);
            int wsplit = 1;
            hipError_t e;
            if (pr.dtype == 0) e = pr.sh == 1 ? launch_strip_wgrad<float, 1>(b, out, &wsplit, st) : launch_strip_wgrad<float, 2>(b, out, &wsplit, st);
            else e = pr.sh == 1 ? launch_strip_wgrad<uint16_t, 1>(b, out, &wsplit, st) : launch_strip_wgrad<uint16_t, 2>(b, out, &wsplit, st);
            if (e != hipSuccess || wsplit == 1) return e;
            dw_reduce_splits_kernel<<<(count + 255) / 256, 256, 0, st>>>(static_cast<const float*>(ws), out, wsplit, count);
            return hipGetLastError();
        }
        DwWArgs a{};
        if (path == WPath::rows) {
            DwRowWArgs r{};
            rows_wgrad_args(pr, in0, in1, r);
            r.out = r.nsplit > 1 ? static_cast<float*>(ws) : out;
            const unsigned grid = (unsigned)(pr.C * r.nsplit);
            if (pr.dtype == 0) {
                if (pr.sh == 1) dw_rows_wgrad_kernel<float, 1><<<grid, 256, 0, st>>>(r);
                else dw_rows_wgrad_kernel<float, 2><<<grid, 256, 0, st>>>(r);
            } else {
                if (pr.sh == 1) dw_rows_wgrad_kernel<uint16_t, 1><<<grid, 256, 0, st>>>(r);
                else dw_rows_wgrad_kernel<uint16_t, 2><<<grid, 256, 0, st>>>(r);
            }
            const hipError_t e = hipGetLastError();
            if (e != hipSuccess || r.nsplit == 1) return e;
            dw_reduce_splits_kernel<<<(count + 255) / 256, 256, 0, st>>>(static_cast<const float*>(ws), out, r.nsplit, count);
            return hipGetLastError();
        }
        wgrad_args(pr, in0, in1, a);
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
    const SPath spath = stencil_path(pass, pr);
    DwStripArgs sa{};
    int stride;
    if (spath == SPath::strip) {
        strip_stencil_args(pass, pr, in0, in1, out, sa, stride);
        sa.bias = pass == 0 ? pr.bias : nullptr;
        sa.mask = pass == 1 ? pr.relu_mask : nullptr;
        sa.dst_bytes = (unsigned)((size_t)sa.planes * sa.OH * sa.OW * sizeof(float));
        if (pr.dtype == 0) return stride == 1 ? launch_strip_stencil<float, 1>(sa, st, fused) : launch_strip_stencil<float, 2>(sa, st, fused);
        return stride == 1 ? launch_strip_stencil<uint16_t, 1>(sa, st, fused) : launch_strip_stencil<uint16_t, 2>(sa, st, fused);
    }
    if (spath == SPath::rows) {
        DwRowArgs ra{};
        bool bwd2;
        rows_args(pass, pr, in0, in1, out, ra, stride, bwd2);
        return pr.dtype == 0 ? launch_rows<float>(ra, stride, bwd2, st) : launch_rows<uint16_t>(ra, stride, bwd2, st);
    }
    if (spath == SPath::none) return hipErrorNotSupported;
    DwArgs a{};
    stencil_args(pass, pr, in0, in1, out, a, stride);
    return pr.dtype == 0 ? launch_stencil<float>(a, stride, st) : launch_stencil<uint16_t>(a, stride, st);
}

}  // namespace miconv
