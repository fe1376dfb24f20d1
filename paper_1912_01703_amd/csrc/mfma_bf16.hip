// Forward and stride-1 backward-data 3x3 convolution of bf16 tensors on the bf16 matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate, fp32 output), gfx950.
//
//   dst[n, f, oh, ow] = sum_{c, r, s} src[n, c, oh-pad_h+r, ow-pad_w+s] * Wt(f, c, r, s)
//   forward        src = x,  Wt(f,c,r,s) = w[f][c][r][s]
//   backward-data  src = dy, Wt(f,c,r,s) = w[c][f][2-r][2-s], pad' = 2-pad
//
// One MFMA contracts 32 reduction channels, and a lane supplies 8 consecutive channels of its
// pixel (B operand) or filter (A operand) as one 16-byte register group.  NCHW keeps a pixel's
// channels a whole plane apart, so two small pre-passes rewrite the operands into the caller's
// workspace with channels innermost: src as [N][H][W][C], the filters as [chunk][tap][f][32 channels]
// (for backward-data already transposed and rotated; a wave's 16 filters are then 1 KB of whole cache lines).  They move each input byte once; the main
// kernel then copies 64-byte runs (32 channels of a pixel) from global memory to LDS and reads
// every operand with one 16-byte access.
//
// Main kernel.  A workgroup owns one image, one 14x14 rectangle of output pixels and 16*FB*WF
// filters and walks the reduction channels in chunks of 32.  Wave (wf, wp) owns 16*FB filters and
// every WP-th 16-pixel block.  Filters live in registers in A-operand layout; the 16x16-pixel
// patch of a chunk sits in LDS as [pixel][32 channels] with 80-byte rows (16-byte reads of 8
// consecutive pixels then fall in distinct banks) and the tap shift is an address immediate.
// One B operand feeds FB MFMAs: LDS bandwidth (128 B/cycle per CU against 4 KB of operands per
// MFMA pair) is what bounds this kernel, not the matrix pipe.
// Everything is pipelined inside the MFMA loop, which holds no vector-ALU instruction: B operands
// are read 7 slots ahead into a ring of 9 register groups, the patch of chunk i+2 is stored to
// its LDS buffer (three buffers) and the registers refilled with chunk i+3, and the filters of
// chunk i+1 replace those of chunk i tap by tap as soon as a tap's MFMAs are issued.
#include "common.h"

namespace miconv {
namespace {

typedef float v2f __attribute__((ext_vector_type(2)));

// Two floats rounded to bf16 (nearest, ties to even; finite values), lo in the low half.
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
    const unsigned a = __float_as_uint(lo), b = __float_as_uint(hi);
    const unsigned ra = (a + 0x7FFFu + ((a >> 16) & 1u)) >> 16, rb = (b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u;
    return ra | rb;
}


// ---- pre-pass 1: [N][C][HW] -> [N][HW][C], 64 channels x 128 pixels per workgroup ----------
// 64 channels are the 128 bytes of one cache line of the destination: a workgroup writes whole lines
// (with 32 channels the two halves of a line came from workgroups on different XCDs).
struct PackXArgs {
    const uint16_t* src;
    uint16_t* dst;
    int N, C, HW;          // C % 32 == 0, HW % 2 == 0 (a plane then starts on a 4-byte boundary)
    unsigned src_bytes;
};

__global__ __launch_bounds__(256) void pack_nhwc_kernel(PackXArgs a) {
    constexpr int LS = 136;   // LDS row stride in elements (16-byte aligned rows)
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * LS];
    const int t = threadIdx.x;
    const int p0 = blockIdx.x * 128, c0 = blockIdx.y * 64, n = blockIdx.z;
    const rsrc_t rs = make_rsrc(a.src, a.src_bytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = t + 256 * i;
        const int c = q >> 4, pc = q & 15;
        // 8 consecutive pixels of one channel (16-byte loads need only 4-byte alignment); the last group of a plane may
        // run into the next plane: those values land in tile columns that no thread reads
        const int p = p0 + 8 * pc;
        const unsigned off = p < a.HW && c0 + c < a.C ? (unsigned)((n * a.C + c0 + c) * a.HW + p) * 2u : kOob;
        const v4u v = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
        *reinterpret_cast<v4u*>(&tile[c * LS + 8 * pc]) = v;
    }
    __syncthreads();
    // thread = (pixel, half of the 64 channels); the two halves of a pixel are waves of this workgroup
    const int px = t & 127, h = t >> 7;
    const int p = p0 + px;
    if (p >= a.HW || c0 + 32 * h >= a.C) return;
    unsigned d[16];
#pragma unroll
    for (int j = 0; j < 16; ++j)
        d[j] = (unsigned)tile[(32 * h + 2 * j) * LS + px] | ((unsigned)tile[(32 * h + 2 * j + 1) * LS + px] << 16);
    v4u* o = reinterpret_cast<v4u*>(a.dst + ((size_t)n * a.HW + p) * a.C + c0 + 32 * h);
#pragma unroll
    for (int j = 0; j < 4; ++j) o[j] = v4u{d[4 * j], d[4 * j + 1], d[4 * j + 2], d[4 * j + 3]};
}

// ---- pre-pass 2: filters -> [tap][f][c] ---------------------------------------------------
struct PackWArgs {
    const uint16_t* w;   // [K][C][3][3]
    uint16_t* dst;       // [Cs/32][9][F][32]: the 32 channels of a chunk are 64 contiguous bytes per (tap, filter)
    int F, Cs, bwd;      // forward: F = K, Cs = C; backward-data: F = C, Cs = K
};

// A workgroup moves 8 filters x one chunk of 32 channels x 9 taps through LDS: contiguous runs on both sides
// (forward: 576 bytes per filter in, 512 bytes per tap out).
__global__ __launch_bounds__(256) void pack_w_kernel(PackWArgs a) {
    __shared__ uint16_t t[8 * 288];   // [filter][channel][tap]
    const int tid = threadIdx.x;
    const int f0 = blockIdx.x * 8, chunk = blockIdx.y, c0 = chunk * 32;
#pragma unroll
    for (int k = 0; k < 9; ++k) {
        const int e = tid + 256 * k;
        if (!a.bwd) {   // w[f][c][tap]: per filter, the chunk's 32 x 9 values are one run
            const int f = e / 288, r = e - f * 288;
            if (f0 + f < a.F) t[e] = a.w[((size_t)(f0 + f) * a.Cs + c0) * 9 + r];
        } else {        // w[c][f][8 - tap]: per reduction channel, the 8 x 9 values of the filters are one run
            const int c = e / 72, r = e - c * 72;
            const int f = r / 9, tap = r - f * 9;
            if (f0 + f < a.F) t[f * 288 + c * 9 + (8 - tap)] = a.w[((size_t)(c0 + c) * a.F + f0) * 9 + r];
        }
    }
    __syncthreads();
    const int f = tid >> 5, c = tid & 31;
    if (f0 + f >= a.F) return;
#pragma unroll
    for (int tap = 0; tap < 9; ++tap)
        a.dst[(((size_t)chunk * 9 + tap) * a.F + f0 + f) * 32 + c] = t[f * 288 + c * 9 + tap];
}

// ---- main kernel ---------------------------------------------------------------------------
struct BfArgs {
    const uint16_t* xt;   // [N][IH][IW][Cs], or (NCHW instances) the source tensor itself, [N][Cs][IH][IW]
    const uint16_t* wp;   // [Cs/32][9][F][32]
    float* dst;           // [N][F][OH][OW]
    int N, Cs, IH, IW, F, OH, OW;
    int pad_h, pad_w;
    int tiles_h, tiles_w, fblocks, units;
    int items;            // work items: units rounded up to a multiple of 8, times fblocks
    int pairs;            // OW is even and dst is 8-byte aligned: the write-out stores two pixels per lane
    int stream_out;       // the result is larger than the 256 MB Infinity Cache: it is stored with the non-temporal hint
    int out_bf16;         // dst holds bf16 (uint16_t) elements: results are rounded to nearest even
};

// The kernel is persistent: a workgroup walks a list of work items (image, tile, filter block), and
// the chunk pipeline runs across item boundaries, so the loads of the next item's first chunks
// overlap the MFMAs of the current one.  Layers with few reduction channels (two chunks per item at
// 64 channels) would otherwise spend most of their time filling and draining the pipeline.
// TH x TW: the tile of output pixels, 14 x 14 or (wide planes) 12 x 16: 12 pixel blocks without a ragged one, and
// output rows of 64 bytes on 64-byte boundaries where 14-pixel rows leave partly written cache lines behind.
// NCHW (12 x 16 tiles only): the source is read as it is, without the channels-innermost copy.  A thread fetches, for
// eight channel planes, the same aligned group of four pixels of a patch row (eight 8-byte loads, the plane chosen by
// the scalar offset; lanes run along the groups of a row), turns the 8 x 4 values into four 16-byte pieces (eight
// channels of one pixel each) with byte permutes right before they are stored to LDS, and stores zeros for pixels
// left or right of the image.  That adds vector-ALU work to the MFMA loop, which a layer bound by HBM (few channels:
// 64 -> 64 at 224 x 224) does not feel, and saves it writing and re-reading a copy of its input.  (Fetching every
// channel of every pixel with a 2-byte load of its own made the texture-address unit the bottleneck: it was busy
// 92 % of the time and the kernel no faster than the copy it replaced.)
template <int TH, int TW, int FB, int WF, int WP, int OCC, bool NCHW = false>
__global__ __launch_bounds__(64 * WF * WP, OCC) void bf16_tile_kernel(BfArgs a) {
    static_assert(!NCHW || TW == 16, "the NCHW gather is laid out for 16-wide tiles");
    constexpr int PH = TH + 2, PW = TW + 2, PSZ = PH * PW, NPX = TH * TW;
    constexpr int NT = 64 * WF * WP;
    constexpr int NB = (NPX + 15) / 16, NBW = (NB + WP - 1) / WP;
    constexpr int ROWB = 80;                 // bytes per patch pixel in LDS: 64 of data, 16 of padding
    // A 16-pixel block of a 14-wide tile wraps to the next patch row.  With this row pitch the
    // wrap continues the 80-byte progression modulo 128 bytes (14 * 80 = 96 mod 128), so the 8 lanes
    // the LDS serves together still hit distinct banks.  A 16-wide tile has one block per row.
    constexpr int RPB = TW == 14 ? 16 * ROWB + 96 : PW * ROWB + 16;
    static_assert((TW == 14 && (RPB - TW * ROWB) % 128 == 0) || (TW == 16 && NPX % 16 == 0), "tile shapes the layout is made for");

    // NCHW: a patch row is covered by GR aligned groups of four pixels; a thread's unit of work is such a group for
    // a quarter of the chunk's 32 channels.
    constexpr int GR = (3 + PW + 3) / 4, NGRP = PH * GR * 4;
    constexpr int XPT = NCHW ? (NGRP + NT - 1) / NT : (PSZ * 4 + NT - 1) / NT;   // pieces (NCHW: groups) per thread and chunk
    // one patch buffer, and room for the pieces that have no place in the patch
    constexpr int BUFB = PH * RPB + (NCHW ? NT : XPT * NT - PSZ * 4) * 16;
    constexpr int NBUF = 3, D = NBUF - 1;
    constexpr int SLOTS = 9 * NBW;           // one slot = one B operand = FB MFMAs
    // B operands are requested PF slots ahead; RING divides SLOTS.  (With a ring of 9 the 14 x 14 instance spilled
    // twelve registers; the NCHW instance holds twice the registers per piece in flight and is not bound by the
    // matrix pipe.)
    constexpr int RING = NCHW ? 6 : (TW == 14 ? 7 : 9), PF = RING - 2;
    static_assert(SLOTS % RING == 0 && PF < RING, "ring");
    constexpr int FW = 16 * FB * WF;         // filters per work item

    __shared__ __attribute__((aligned(16))) unsigned char xs[NBUF * BUFB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = wave % WF, wp = wave / WF;
    const int li = lane & 15, kk = lane >> 4;
    const int nchunks = a.Cs / 32;
    const int plane = a.IH * a.IW;
    const unsigned plane_bytes = (unsigned)plane * 2u;
    const unsigned img_bytes = (unsigned)(a.IH * a.IW * a.Cs) * 2u;
    const unsigned tap_bytes = (unsigned)a.F * 64u;
    const int tiles = a.tiles_h * a.tiles_w;

    // Work item j of this workgroup is number blockIdx.x + j * gridDim.x (gridDim.x is a multiple of 8).
    // Consecutive numbers land on different XCDs; the filter blocks of one (image, tile) are given
    // numbers that differ by multiples of 8, run at about the same time and share an L2.
    const int nitems = __builtin_amdgcn_readfirstlane(a.items > (int)blockIdx.x ? (a.items - 1 - (int)blockIdx.x) / (int)gridDim.x + 1 : 0);
    struct Item { int ok, fblk, n, oh0, ow0; };
    auto item = [&](int j) __attribute__((always_inline)) -> Item {
        Item it{0, 0, 0, 0, 0};
        if (j >= nitems) return it;
        const int w = blockIdx.x + j * gridDim.x;
        const int xcd = w & 7, rest = w >> 3;
        it.fblk = rest % a.fblocks;
        // every XCD owns a contiguous run of units: neighbouring tiles, whose 56-byte output rows and input halos share
        // cache lines, then go through the same L2 at about the same time (layer 4a: 860 -> 784 us; one workgroup
        // taking a run of neighbouring tiles by itself was slower, 929 us)
        const int unit = __builtin_amdgcn_readfirstlane(xcd * ((a.units + 7) >> 3) + rest / a.fblocks);
        if (unit >= a.units) return it;
        // integer division goes through the vector ALU: tell the compiler the results are wave-uniform
        const int t = unit % tiles;
        it.ok = 1;
        it.fblk = __builtin_amdgcn_readfirstlane(it.fblk);
        it.n = __builtin_amdgcn_readfirstlane(unit / tiles);
        it.oh0 = __builtin_amdgcn_readfirstlane((t / a.tiles_w) * TH);
        it.ow0 = __builtin_amdgcn_readfirstlane((t % a.tiles_w) * TW);
        return it;
    };

    // ---- the three positions of the pipeline ---------------------------------------------------------
    // patch loads run D+1 chunks ahead of the MFMAs, filter loads one chunk ahead
    int xj = 0, xch = 0;            // item and chunk the next patch load fetches
    unsigned goff[XPT];             // its gather plan: piece = (pixel, quarter of the chunk's 32 channels)
    unsigned gin[NCHW ? XPT : 1];   // NCHW: which pixels of a group lie inside the image
    // NCHW: a group's first pixel lies D0 pixels left of the patch's first column (pad 0: 0, pad 1: 3, pad 2: 2)
    const int D0 = (4 - a.pad_w) & 3;
    int loff[NCHW ? 1 : XPT];       // where a piece goes in a patch buffer
    int loffk[NCHW ? XPT : 1][4];   // NCHW: where the four pixels of a group go; pixels outside the patch go to a spare slot
#pragma unroll
    for (int m = 0; m < XPT; ++m) {
        const int e = tid + NT * m;
        if constexpr (NCHW) {
            const int q = e / (PH * GR), r = e - q * (PH * GR);
            const int ph = r / GR, g = r - ph * GR;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int pw = 4 * g + k - D0;
                loffk[m][k] = e < NGRP && pw >= 0 && pw < PW ? ph * RPB + pw * ROWB + q * 16 : PH * RPB + tid * 16;
            }
        } else {
            const int pix = e >> 2, q = e & 3;
            loff[m] = pix < PSZ ? (pix / PW) * RPB + (pix % PW) * ROWB + q * 16 : PH * RPB + (e - PSZ * 4) * 16;
        }
    }

    const uint16_t* xsrc = a.xt;
    int xok = 0;
    auto plan_patch = [&]() __attribute__((always_inline)) {
        const Item it = item(xj);
        xok = it.ok;
        xsrc = a.xt + (size_t)it.n * a.IH * a.IW * a.Cs;
        const int ih0 = it.oh0 - a.pad_h, iw0 = it.ow0 - a.pad_w;
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int e = tid + NT * m;
            if constexpr (NCHW) {
                // group e = (quarter q of the channels, patch row ph, group g of the row); the row's first group starts
                // at the multiple of four at or below its first pixel (tile origins are multiples of 16)
                const int q = e / (PH * GR), r = e - q * (PH * GR);
                const int ph = r / GR, g = r - ph * GR;
                const int ih = ih0 + ph, iwg = iw0 - D0 + 4 * g;
                const bool ok = e < NGRP && ih >= 0 && ih < a.IH;
                // (a group that starts left of the row may start before the descriptor: the offset wraps and reads zeros)
                goff[m] = ok ? (unsigned)(8 * q * plane + ih * a.IW + iwg) * 2u : kOob;
                unsigned inside = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) inside |= (iwg + k >= 0 && iwg + k < a.IW ? 1u : 0u) << k;
                gin[m] = inside;
            } else {
                const int pix = e >> 2, q = e & 3;
                const int ph = pix / PW, pw = pix - ph * PW;
                const int ih = ih0 + ph, iw = iw0 + pw;
                const bool ok = pix < PSZ && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
                goff[m] = ok ? (unsigned)((ih * a.IW + iw) * a.Cs + 8 * q) * 2u : kOob;
            }
        }
    };
    auto patch_rsrc = [&]() __attribute__((always_inline)) -> rsrc_t {   // past the last item: reads zeros
        if constexpr (NCHW) return make_rsrc(xsrc + (size_t)xch * 32 * plane, xok ? 32u * plane_bytes : 0u);
        else return make_rsrc(xsrc + xch * 32, xok ? img_bytes - (unsigned)xch * 64u : 0u);
    };
    // What a thread holds of a chunk's patch between its loads and its LDS stores: 16-byte pieces, or (NCHW) per group
    // the eight 8-byte values (four pixels of eight channel planes) and which of the four pixels lie inside the image.
    struct Held {
        v4u v[NCHW ? 1 : XPT];
        v2u raw[NCHW ? XPT : 1][8];
        unsigned inside[NCHW ? XPT : 1];
    };
    auto load_patch = [&](Held& h, const rsrc_t& xrs, int m) __attribute__((always_inline)) {
        if constexpr (NCHW) {
            // (a valid group has all eight planes inside the descriptor; an invalid one carries kOob in its vector offset)
#pragma unroll
            for (int j = 0; j < 8; ++j) h.raw[m][j] = __builtin_amdgcn_raw_buffer_load_b64(xrs, goff[m], j * plane_bytes, 0);
            h.inside[m] = gin[m];
        } else {
            h.v[m] = __builtin_amdgcn_raw_buffer_load_b128(xrs, goff[m], 0, 0);
        }
    };
    auto store_patch = [&](const Held& h, unsigned char* buf, int m) __attribute__((always_inline)) {
        if constexpr (NCHW) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {   // pixel k of the group: channels 2i, 2i+1 are the halves k%2 of dword k/2 of planes 2i, 2i+1
                v4u piece;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const unsigned both = __builtin_amdgcn_perm(h.raw[m][2 * i + 1][k / 2], h.raw[m][2 * i][k / 2], k % 2 ? 0x07060302u : 0x05040100u);
                    piece[i] = (h.inside[m] >> k) & 1u ? both : 0u;
                }
                *reinterpret_cast<v4u*>(buf + loffk[m][k]) = piece;
            }
        } else {
            *reinterpret_cast<v4u*>(buf + loff[m]) = h.v[m];
        }
    };
    auto advance_patch = [&]() __attribute__((always_inline)) {
        if (++xch == nchunks) { xch = 0; ++xj; plan_patch(); }
    };
    int wj = 0, wch = 0;            // item and chunk the next filter load fetches
    unsigned wofs[FB];              // this lane's filter rows: filter f, channels 8*kk .. 8*kk+7 of the chunk (tap 0)
    int wok = 0;
    auto plan_filters = [&]() __attribute__((always_inline)) {
        const Item it = item(wj);
        wok = it.ok;
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
            const int f = it.fblk * FW + wf * (16 * FB) + 16 * fb + li;
            wofs[fb] = f < a.F ? (unsigned)(f * 32 + 8 * kk) * 2u : kOob;
        }
    };
    auto filter_rsrc = [&]() __attribute__((always_inline)) -> rsrc_t {
        const unsigned chunk_bytes = 9u * tap_bytes;
        return make_rsrc(reinterpret_cast<const unsigned char*>(a.wp) + (size_t)wch * chunk_bytes, wok ? chunk_bytes : 0u);
    };
    auto advance_filters = [&]() __attribute__((always_inline)) {
        if (++wch == nchunks) { wch = 0; ++wj; plan_filters(); }
    };

    // B operand addresses of this lane's pixel in each of its blocks (tap (0,0), buffer 0)
    int pixb[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        int j = 16 * (wp + WP * i) + li;
        if (j >= NPX) j = 0;   // padding lanes read a valid address; their results are never stored
        const int th = j / TW, tw = j - th * TW;
        pixb[i] = th * RPB + tw * ROWB + kk * 16;
    }
    const bool last_ok = wp + WP * (NBW - 1) < NB;   // does this wave own a block in its last slot?
    auto mine = [&](int i) __attribute__((always_inline)) -> bool { return !(NB % WP != 0 && i == NBW - 1 && !last_ok); };
    auto tapoff = [](int tap) { return (tap / 3) * RPB + (tap % 3) * ROWB; };

    v4f acc[FB][NBW];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb)
#pragma unroll
        for (int i = 0; i < NBW; ++i) acc[fb][i] = v4f{0.f, 0.f, 0.f, 0.f};
    v4u A[9][FB];
    Held xreg;
    v4u ring[RING];

    if (nitems == 0) return;
    // ---- prologue: filters of the first chunk; patches of chunks 0..D-1 to LDS, chunk D to registers ----
    plan_patch();
    plan_filters();
    {
        const rsrc_t wrs = filter_rsrc();
#pragma unroll
        for (int tap = 0; tap < 9; ++tap)
#pragma unroll
            for (int fb = 0; fb < FB; ++fb) A[tap][fb] = __builtin_amdgcn_raw_buffer_load_b128(wrs, wofs[fb], tap * tap_bytes, 0);
        advance_filters();
        // the patches of chunks 0..D are all requested before the first one is waited for
        Held pre[D];
#pragma unroll
        for (int c = 0; c < D; ++c) {
            const rsrc_t xrs = patch_rsrc();
#pragma unroll
            for (int m = 0; m < XPT; ++m) load_patch(pre[c], xrs, m);
            advance_patch();
        }
        {
            const rsrc_t xrs = patch_rsrc();
#pragma unroll
            for (int m = 0; m < XPT; ++m) load_patch(xreg, xrs, m);
            advance_patch();
        }
#pragma unroll
        for (int c = 0; c < D; ++c)
#pragma unroll
            for (int m = 0; m < XPT; ++m) store_patch(pre[c], xs + c * BUFB, m);
        __syncthreads();
#pragma unroll
        for (int s = 0; s < PF; ++s)
            if (mine(s % NBW)) ring[s % RING] = *reinterpret_cast<const v4u*>(xs + pixb[s % NBW] + tapoff(s / NBW));
    }

    int rd = 0, nx = BUFB, wr = D * BUFB;
    int cj = 0, cch = 0;            // item and chunk being multiplied
    const int total = nitems * nchunks;
    for (int g = 0; g < total; ++g) {
        const rsrc_t xrs = patch_rsrc();
        const rsrc_t wrs = filter_rsrc();
        const unsigned char* pr[NBW];
        const unsigned char* pn[NBW];
#pragma unroll
        for (int i = 0; i < NBW; ++i) { pr[i] = xs + rd + pixb[i]; pn[i] = xs + nx + pixb[i]; }
        unsigned char* const pw = xs + wr;
        unsigned char* ps[NCHW ? 1 : XPT];
        if constexpr (!NCHW) {
#pragma unroll
            for (int m = 0; m < XPT; ++m) ps[m] = pw + loff[m];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < SLOTS; ++s) {
            const int tap = s / NBW, i = s % NBW;
            {   // request the B operand of slot s + PF (of the next chunk's buffer past the end of this one)
                const int s2 = s + PF;
                const int t2 = (s2 % SLOTS) / NBW, i2 = s2 % NBW;
                if (mine(i2)) {
                    const unsigned char* base = s2 < SLOTS ? pr[i2] : pn[i2];
                    ring[s2 % RING] = *reinterpret_cast<const v4u*>(base + tapoff(t2));
                }
            }
            if (mine(i)) {
#pragma unroll
                for (int fb = 0; fb < FB; ++fb)
                    acc[fb][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, A[tap][fb]),
                                                                         __builtin_bit_cast(v8bf, ring[s % RING]),
                                                                         acc[fb][i], 0, 0, 0);
            }
            // patch D chunks ahead: registers -> LDS in the last third of the slots, and right behind each store the
            // load of the chunk after it refills the same registers, which gives a load a whole chunk to arrive
#pragma unroll
            for (int m = 0; m < XPT; ++m) {
                if (2 * SLOTS / 3 + m * (SLOTS / 3) / XPT == s) {
                    if constexpr (NCHW) store_patch(xreg, pw, m);
                    else *reinterpret_cast<v4u*>(ps[m]) = xreg.v[m];
                    load_patch(xreg, xrs, m);
                }
            }
            // this tap's filters are no longer needed: fetch the next chunk's into the same registers
            if (i == NBW - 1) {
#pragma unroll
                for (int fb = 0; fb < FB; ++fb) A[tap][fb] = __builtin_amdgcn_raw_buffer_load_b128(wrs, wofs[fb], tap * tap_bytes, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        advance_patch();
        advance_filters();
        if (++cch == nchunks) {
            // ---- the item is complete: D[f = 4*kk+v][pixel = li] to memory, accumulators back to zero ----
            const Item it = item(cj);
            const int dplane = a.OH * a.OW;
            float* dst = a.dst + (size_t)it.n * a.F * dplane;
            const int fbase = it.fblk * FW + wf * (16 * FB);
            if (a.out_bf16) {
                // bf16 results: after the same trade between neighbouring lanes a lane packs its two pixels of a filter
                // into one 4-byte store (rows of an even number of pixels), else every value is a 2-byte store
                uint16_t* dst16 = reinterpret_cast<uint16_t*>(a.dst) + (size_t)it.n * a.F * dplane;
                const bool odd = li & 1;
#pragma unroll
                for (int i = 0; i < NBW; ++i) {
                    const int j = 16 * (wp + WP * i) + li;
                    const int th = j / TW, tw = j - th * TW;
                    const int oh = it.oh0 + th, ow = it.ow0 + tw;
                    const bool pix_ok = it.ok && j < NPX && oh < a.OH && ow < a.OW;
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) {
                        const v4f c = acc[fb][i];
                        if (a.pairs) {
                            const float s0 = odd ? c[0] : c[2], s1 = odd ? c[1] : c[3];
                            const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s0), 0xB1, 0xF, 0xF, true));
                            const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s1), 0xB1, 0xF, 0xF, true));
                            const unsigned o0 = odd ? pack_bf16(r0, c[2]) : pack_bf16(c[0], r0);
                            const unsigned o1 = odd ? pack_bf16(r1, c[3]) : pack_bf16(c[1], r1);
                            const int f = fbase + 16 * fb + 4 * kk + (odd ? 2 : 0);
                            uint16_t* row = dst16 + (size_t)f * dplane + oh * a.OW + (ow - (odd ? 1 : 0));
                            if (pix_ok && f < a.F) *reinterpret_cast<unsigned*>(row) = o0;
                            if (pix_ok && f + 1 < a.F) *reinterpret_cast<unsigned*>(row + dplane) = o1;
                        } else {
#pragma unroll
                            for (int v = 0; v < 4; ++v) {
                                const int f = fbase + 16 * fb + 4 * kk + v;
                                if (pix_ok && f < a.F) dst16[(size_t)f * dplane + oh * a.OW + ow] = static_cast<uint16_t>(pack_bf16(c[v], 0.f));
                            }
                        }
                        acc[fb][i] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
            } else if (a.pairs) {
                // Neighbouring lanes hold neighbouring pixels of one row (tile width, block size and tile origin
                // are even).  They trade two of their four filters, after which the even lane owns filters
                // 4kk, 4kk+1 and the odd lane 4kk+2, 4kk+3 of both pixels: 8-byte stores, half as many.
                const bool odd = li & 1;
#pragma unroll
                for (int i = 0; i < NBW; ++i) {
                    const int j = 16 * (wp + WP * i) + li;
                    const int th = j / TW, tw = j - th * TW;
                    const int oh = it.oh0 + th, ow = it.ow0 + tw;
                    const bool pix_ok = it.ok && j < NPX && oh < a.OH && ow < a.OW;   // the same for both lanes of a pair
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) {
                        const v4f c = acc[fb][i];
                        const float s0 = odd ? c[0] : c[2], s1 = odd ? c[1] : c[3];
                        const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s0), 0xB1, 0xF, 0xF, true));
                        const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, s1), 0xB1, 0xF, 0xF, true));
                        const float2 o0 = odd ? make_float2(r0, c[2]) : make_float2(c[0], r0);
                        const float2 o1 = odd ? make_float2(r1, c[3]) : make_float2(c[1], r1);
                        const int f = fbase + 16 * fb + 4 * kk + (odd ? 2 : 0);
                        float* row = dst + (size_t)f * dplane + oh * a.OW + (ow - (odd ? 1 : 0));
                        if (a.stream_out) {   // (567 -> 539 us on 64 -> 64 channels at 224 x 224, N = 64)
                            if (pix_ok && f < a.F) __builtin_nontemporal_store(v2f{o0.x, o0.y}, reinterpret_cast<v2f*>(row));
                            if (pix_ok && f + 1 < a.F) __builtin_nontemporal_store(v2f{o1.x, o1.y}, reinterpret_cast<v2f*>(row + dplane));
                        } else {
                            if (pix_ok && f < a.F) *reinterpret_cast<float2*>(row) = o0;
                            if (pix_ok && f + 1 < a.F) *reinterpret_cast<float2*>(row + dplane) = o1;
                        }
                        acc[fb][i] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
            } else {
#pragma unroll
                for (int i = 0; i < NBW; ++i) {
                    const int j = 16 * (wp + WP * i) + li;
                    const int th = j / TW, tw = j - th * TW;
                    const int oh = it.oh0 + th, ow = it.ow0 + tw;
                    const bool pix_ok = it.ok && j < NPX && oh < a.OH && ow < a.OW;
#pragma unroll
                    for (int fb = 0; fb < FB; ++fb) {
#pragma unroll
                        for (int v = 0; v < 4; ++v) {
                            const int f = fbase + 16 * fb + 4 * kk + v;
                            if (pix_ok && f < a.F) dst[(size_t)f * dplane + oh * a.OW + ow] = acc[fb][i][v];
                        }
                        acc[fb][i] = v4f{0.f, 0.f, 0.f, 0.f};
                    }
                }
            }
            cch = 0;
            ++cj;
        }
        __syncthreads();
        rd = nx;
        nx = nx + BUFB == NBUF * BUFB ? 0 : nx + BUFB;
        wr = wr + BUFB == NBUF * BUFB ? 0 : wr + BUFB;
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // loads fetched past the last chunk still target registers
}

// 32 filters per wave (one B operand feeds two MFMAs), 2 x 2 waves, two workgroups per CU.  Wider waves
// (64 filters, or all 13 pixel blocks) spill; four pixel-block waves leave too few MFMAs per chunk.
constexpr int kFB = 2, kWF = 2, kWP = 2, kOCC = 2;

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Shape {
    int Cs, F, IH, IW, OH, OW, pad_h, pad_w;
};

// Layers with few reduction channels on wide planes are bound by HBM, not by the matrix cores: they read the source
// tensor as it is (the NCHW instance of the kernel, 12 x 16 tiles) instead of writing and re-reading a channels-innermost
// copy of it.  Its 8-byte loads of four pixels need rows of an even number of pixels.
bool reads_nchw(const Shape& s) { return s.Cs <= 128 && s.OW % 16 == 0 && s.OH >= 96 && s.IW % 2 == 0; }

bool shape_of(int pass, const Problem& pr, Shape& s) {
    if (pr.dtype != 1 || pr.R != 3 || pr.S != 3 || pr.sh != 1 || pr.sw != 1 || pr.groups != 1) return false;
    if (pr.ph > 2 || pr.pw > 2) return false;
    if (pass == 0) s = Shape{pr.C, pr.K, pr.H, pr.W, pr.P, pr.Q, pr.ph, pr.pw};
    else if (pass == 1) s = Shape{pr.K, pr.C, pr.P, pr.Q, pr.H, pr.W, 2 - pr.ph, 2 - pr.pw};
    else return false;
    if (s.Cs % 32 != 0 || (s.IH * s.IW) % 2 != 0) return false;   // (planes of an even number of pixels start 4-byte aligned)
    const size_t lim = (size_t)1 << 31;
    if ((size_t)pr.N * s.Cs * s.IH * s.IW * 2 >= lim || (size_t)pr.N * s.F * s.OH * s.OW * 4 >= ((size_t)1 << 33)) return false;
    if ((size_t)9 * s.F * s.Cs * 2 >= lim) return false;
    return true;
}

}  // namespace

bool bf16_tile_supports(int pass, const Problem& pr) {
    Shape s;
    return shape_of(pass, pr, s);
}

bool bf16_tile_accepts(int pass, const Problem& pr, const void* in0) {
    Shape s;
    return shape_of(pass, pr, s) && reinterpret_cast<uintptr_t>(in0) % 4 == 0;
}

size_t bf16_tile_workspace_bytes(int pass, const Problem& pr) {
    Shape s;
    if (!shape_of(pass, pr, s)) return 0;
    // (the copy is not used when the NCHW instance runs, but whether it does also depends on the source's alignment,
    // which the query does not know: tensors that are at least 4-byte aligned need the packed filters only)
    return round256((size_t)9 * s.F * s.Cs * 2) + (reads_nchw(s) ? 0 : round256((size_t)pr.N * s.IH * s.IW * s.Cs * 2));
}

hipError_t bf16_tile_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                         hipStream_t st) {
    Shape s;
    if (!shape_of(pass, pr, s)) return hipErrorNotSupported;
    // workspace: the packed filters first, then (if made) the channels-innermost copy of the source
    if (reinterpret_cast<uintptr_t>(in0) % 4 != 0) return hipErrorNotSupported;   // every path here loads 4 bytes and more at a time
    const bool nchw = reads_nchw(s);
    uint16_t* wp = static_cast<uint16_t*>(ws);
    const uint16_t* xt = static_cast<const uint16_t*>(in0);
    const int HW = s.IH * s.IW;
    hipError_t e = hipSuccess;
    if (!nchw) {
        uint16_t* copy = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(ws) + round256((size_t)9 * s.F * s.Cs * 2));
        PackXArgs px{static_cast<const uint16_t*>(in0), copy, pr.N, s.Cs, HW, (unsigned)((size_t)pr.N * s.Cs * HW * 2)};
        pack_nhwc_kernel<<<dim3((HW + 127) / 128, (s.Cs + 63) / 64, pr.N), 256, 0, st>>>(px);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        xt = copy;
    }

    PackWArgs pw{static_cast<const uint16_t*>(in1), wp, s.F, s.Cs, pass == 1 ? 1 : 0};
    pack_w_kernel<<<dim3((s.F + 7) / 8, s.Cs / 32), 256, 0, st>>>(pw);
    e = hipGetLastError();
    if (e != hipSuccess) return e;

    BfArgs a{};
    a.xt = xt; a.wp = wp; a.dst = out;
    a.N = pr.N; a.Cs = s.Cs; a.IH = s.IH; a.IW = s.IW; a.F = s.F; a.OH = s.OH; a.OW = s.OW;
    a.pad_h = s.pad_h; a.pad_w = s.pad_w;
    const bool wide = s.OW % 16 == 0 && s.OH >= 96;   // 12 x 16 tiles
    const int th = wide ? 12 : 14, tw = wide ? 16 : 14;
    a.tiles_h = (s.OH + th - 1) / th; a.tiles_w = (s.OW + tw - 1) / tw;
    a.fblocks = (s.F + 16 * kFB * kWF - 1) / (16 * kFB * kWF);
    a.units = pr.N * a.tiles_h * a.tiles_w;
    a.items = ((a.units + 7) / 8) * 8 * a.fblocks;
    a.out_bf16 = pr.out_bf16 ? 1 : 0;
    // two pixels per store: rows of an even number of pixels, and a result aligned to one such store
    a.pairs = s.OW % 2 == 0 && reinterpret_cast<uintptr_t>(out) % (pr.out_bf16 ? 4 : 8) == 0;
    a.stream_out = !pr.out_bf16 && (size_t)pr.N * s.F * s.OH * s.OW * sizeof(float) > ((size_t)256 << 20);
    // two workgroups fit a CU: at most that many are launched and each walks its share of the items
    const int grid = a.items < 256 * kOCC ? a.items : 256 * kOCC;
    if (nchw) bf16_tile_kernel<12, 16, kFB, kWF, kWP, kOCC, true><<<grid, 64 * kWF * kWP, 0, st>>>(a);
    else if (wide) bf16_tile_kernel<12, 16, kFB, kWF, kWP, kOCC><<<grid, 64 * kWF * kWP, 0, st>>>(a);
    else bf16_tile_kernel<14, 14, kFB, kWF, kWP, kOCC><<<grid, 64 * kWF * kWP, 0, st>>>(a);
    return hipGetLastError();
}

}  // namespace miconv
