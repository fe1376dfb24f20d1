// Kernel template shared by mfma_tile.hip (forward, stride-1 backward-data) and
// mfma_tile_phase.hip (strided backward-data, one launch per output phase).
#pragma once
// Forward and stride-1 backward-data convolution as an implicit GEMM on the
// fp32 matrix cores (v_mfma_f32_16x16x4_f32), written for gfx950.
//
// Both passes are the same computation on different operands:
//   dst[n, g*Fg+f, oh, ow] = sum_{c<Rg, r, s} src[n, g*Rg+c, oh*ST-pad_h+r, ow*ST-pad_w+s] * Wt(f,c,r,s)
//   forward        src = x,  dst = y,  Wt(f,c,r,s) = w[g*Fg+f][c][r][s]
//   backward-data  src = dy, dst = dx, Wt(f,c,r,s) = w[g*Rg+c][f][R-1-r][S-1-s], pad' = R-1-pad (stride 1)
//
// Decomposition.  A workgroup owns one image, one TH x TW rectangle of output
// pixels and 16*WF filters, and walks the reduction channels in chunks of CK.
//   * The source patch a chunk needs ((TH-1)*ST+R rows, (TW-1)*ST+S columns, CK
//     channels, zero-filled outside the image) is gathered once into LDS with
//     coalesced row reads; the R*S-fold reuse of every input value (the im2col
//     expansion) only ever happens as LDS reads at a per-tap address offset.
//   * Filter values go straight from global memory into registers in the MFMA
//     A-operand layout (each wave owns 16 filters, so there is nothing to share).
//   * MFMA roles: M = 16 filters, N = 16 output pixels, K = 4 reduction channels.
//     Lane l holds A[f = l%16][k = l/16], B[k = l/16][pixel = l%16] and
//     D[f = 4*(l/16)+v][pixel = l%16] in accumulator register v.
//   * The patch is pipelined through NBUF LDS buffers entirely inside the MFMA loop: while chunk i
//     is multiplied, the registers that hold the patch of chunk i+NBUF-1 (loaded during chunk i-1)
//     are stored to its buffer, then refilled with the loads of chunk i+NBUF; the filters of chunk
//     i+1 are loaded into the second register set.  One barrier per chunk and no separate copy phase.
//     With three buffers the next chunk's patch was complete a barrier earlier, so the first LDS
//     operands of chunk i+1 are requested before the barrier and the MFMA stream runs through it;
//     the launchers nevertheless use two (shorter start-up, less LDS), which measured faster.
//   * An ordinary vector instruction does not overlap with a running MFMA of its own SIMD, so the
//     loop holds only MFMAs, LDS accesses, loads and waits: every address is a register prepared
//     outside the loop plus an immediate.
#include "common.h"
#include <type_traits>

namespace miconv {
namespace tile {


struct TileArgs {
    const void* src;
    const void* wgt;
    float* dst;
    int N, Csrc, IH, IW;   // source tensor [N][Csrc][IH][IW]
    int Cdst, OH, OW;      // destination tensor [N][Cdst][OH][OW]
    int Fg, Rg, groups;    // destination / reduction channels per group
    int pad_h, pad_w;      // source row = oh*ST - pad_h + r
    int tiles_h, tiles_w;  // spatial tiles per image
    int fblocks;           // filter blocks per group
    int units;             // N * groups * tiles_h * tiles_w
    unsigned wgt_bytes;    // size of the filter tensor
    // Strided backward-data runs once per output phase (see mfma_tile_phase.hip): the kernel then
    // computes a stride-1 correlation of dy with a sub-filter and writes every o_s-th output pixel.
    int o_sh, o_sw;        // destination pixel (oh, ow) of the phase grid is row oh*o_sh + o_oh, column ow*o_sw + o_ow
    int o_oh, o_ow;
    int DH, DW;            // full destination plane
    int w_rs;              // taps of the full filter (R*S of the layer)
    int tapoff[9];         // phase mode: offset of sub-filter tap t inside a (k, c) filter plane
    int items;             // work item ids: units rounded up to a multiple of 8, times fblocks
    int fill2;             // phase mode, 1x1 filter at stride 2: the three pixels next to every written one get zeros
    // Fused epilogues of the write-out (both null: plain convolution).
    const float* bias;     // [Cdst]: dst = max(0, dst + bias[channel])
    const void* mask;      // shaped and typed like the destination's counterpart among the inputs: dst = mask > 0 ? dst : 0
};

// Smallest channel stride >= v such that kq consecutive channels span 16 banks (mod 32): the two
// lane groups of a half-wave, which are kq channels apart, then read disjoint halves of the 32 LDS banks.
constexpr int lds_channel_stride(int v, int kq) {
    while ((v * kq) % 32 != 16) ++v;
    return v;
}

// T: element type of src and wgt (float, or uint16_t holding bf16).
// R,S: filter size.  ST: stride.  TH,TW: output tile.  CK: channels per chunk (4, 8, 16 or 32).
// WF: waves along filters (16 filters each).  WP: waves along pixel blocks.  BWD: backward-data operand mapping.
// WV: the reduction channels per group are a multiple of 4 (forward filters can be read four values at a time).
// PHASE: one output phase of a strided backward-data pass (R, S are the sub-filter's size; BWD is set).
// NBUF: LDS patch buffers (2 or 3).
// PERSIST: the grid is smaller than the number of work items; a workgroup walks items blockIdx.x,
//     blockIdx.x + gridDim.x, ... and the chunk pipeline runs across item boundaries, so that the
//     start-up loads and the write-out of one item overlap the MFMAs of its neighbours (layers with
//     few chunks per item and many items).
// MERGE2: backward-data of a 3x3 stride-2 padding-1 layer in one launch (BWD set, R = S = 3, ST = 1).  Output
//     pixel (h, v) belongs to phase (a, b) = ((h+1) % 2, (v+1) % 2) and only taps r = a (mod 2), s = b (mod 2)
//     reach it, so the nine taps of the filter split over four accumulator sets that all read the same dy
//     patch: a work item is a 14x14 rectangle of the half-resolution grid (28x28 dx pixels).  With
//     h = 2*i + 1 - a for grid row i, tap r reads dy row i + (r == 0), see roff() below.
// XW: the patch is TH full rows of the source plane (1x1 filter, no padding, tile as wide as the plane) and planes are
//     multiples of 16 bytes: a chunk's patch is then one contiguous run of CK planes, read 16 bytes per lane.
template <typename T, int R, int S, int ST, int TH, int TW, int CK, int WF, int WP, bool BWD, bool WV, bool PHASE, int NBUF = 2,
          bool XW = false, bool PERSIST = false, bool MERGE2 = false>
__global__ __launch_bounds__(64 * WF * WP) void conv_tile_kernel(TileArgs a) {
    constexpr int NT = 64 * WF * WP;
    constexpr int RS = R * S;
    static_assert(!MERGE2 || (BWD && !PHASE && !XW && R == 3 && S == 3 && ST == 1), "merged stride-2 backward-data");
    // A strided 1x1 filter only ever reads the pixels (oh*ST, ow*ST): the patch holds just those (SPARSE), not the
    // (TH-1)*ST+1 rows and columns between them.
    constexpr bool SPARSE = R == 1 && S == 1 && ST > 1 && !MERGE2;
    constexpr int PST = SPARSE ? 1 : ST;     // pixel stride inside the LDS patch
    constexpr int GST = SPARSE ? ST : 1;     // source stride between neighbouring patch elements
    constexpr int PH = MERGE2 ? TH + 1 : (TH - 1) * PST + R, PW = MERGE2 ? TW + 1 : (TW - 1) * PST + S;
    constexpr int PSZ = PH * PW;
    constexpr int KQ = CK / 4;  // channels per lane group: lane group kk owns channels [kk*KQ, kk*KQ+KQ) of a chunk
    static_assert(CK == 4 || CK == 8 || CK == 16 || CK == 32 || CK == 64, "CK must be 4, 8, 16, 32 or 64");
    static_assert(!XW || (R == 1 && S == 1 && ST == 1 && PSZ % 4 == 0 && sizeof(T) == 4), "whole-plane patches only");
    constexpr int CS = lds_channel_stride(PSZ, KQ);
    constexpr int XE = CK * PSZ;
    constexpr int XPT = XW ? (XE / 4 + NT - 1) / NT : (XE + NT - 1) / NT;   // load pieces per thread
    constexpr int NPX = TH * TW;
    constexpr int NB = (NPX + 15) / 16;      // 16-pixel blocks in the tile
    // A last block of at most four pixels (196 = 12 * 16 + 4) is not run as a 16 x 16 x 4 MFMA with twelve idle
    // columns: v_mfma_f32_4x4x1_16B_f32 (sixteen independent 4 x 4 x 1 products, a quarter of the time) takes it,
    // block b = 4 * kq + fg of the instruction being filters 4 * fg .. + 3 times the four pixels for the reduction
    // channel of lane group kq.  Lane l = 4 * b + i is row i of block b for A and column i for B, which is the layout
    // the filter registers already have (filter l % 16, lane group l / 16); the B operand is the pixel l % 4.  The
    // four partial sums per (filter, pixel) are added and moved to the 16 x 16 layout once, before the write-out.
    // Only where every wave keeps at least two full blocks: on 7 x 7 tiles (three full blocks for two waves) the wave
    // left with one MFMA per group no longer covers its LDS reads (3x3, 512 channels: forward 173 -> 201 us).
    constexpr int RAG = NPX % 16;
    constexpr bool QUAD = RAG >= 1 && RAG <= 4 && (NB - 1) >= 2 * WP;
    // Block slots of a wave: the full blocks are dealt out to the WP waves in turn (wave wp, slot i: block wp + WP * i),
    // and the small last block has a slot of its own behind them, which belongs to wave 0.  So a slot is of one kind
    // for every wave, and what differs between waves is only whether they own it (a wave-uniform skip).
    constexpr int NBF = QUAD ? NB - 1 : NB;                  // blocks run as 16 x 16 x 4
    constexpr int NBWF = (NBF + WP - 1) / WP;                // their slots
    constexpr int NBW = NBWF + (QUAD ? 1 : 0);               // slots per wave

    static_assert(NBUF == 2 || NBUF == 3, "two or three patch buffers");
    // Each buffer is followed by 64 words that lanes without an element store to (no branch around a
    // store that sits between MFMAs).
    constexpr int BUFSZ = ((CK * CS + 3) & ~3) + 64, TRASH = BUFSZ - 64;
    __shared__ float xs[NBUF * BUFSZ];

    // ---- which unit of work -------------------------------------------------------------
    // Consecutive workgroup ids land on different XCDs (8 of them, one L2 each).  All filter
    // blocks of one (image, tile) are given ids that differ by multiples of 8 so that they share an L2.
    struct Item { int ok, fblk, n, g, oh0, ow0; };
    auto decode = [&](int b) __attribute__((always_inline)) -> Item {
        Item it{0, 0, 0, 0, 0, 0};
        const int xcd = b & 7;
        const int rest = b >> 3;
        it.fblk = __builtin_amdgcn_readfirstlane(rest % a.fblocks);
        // every XCD owns a contiguous run of units: neighbouring tiles, whose output rows and input halos share cache
        // lines, go through the same L2 at about the same time (224x224 planes: forward 2120 -> 2005 us)
        const int unit = __builtin_amdgcn_readfirstlane(xcd * ((a.units + 7) >> 3) + rest / a.fblocks);
        if (b >= a.items || unit >= a.units) return it;
        // (integer division goes through the vector ALU: readfirstlane tells the compiler the results are wave-uniform)
        int u = unit;
        const int tj = u % a.tiles_w; u /= a.tiles_w;
        const int ti = u % a.tiles_h; u /= a.tiles_h;
        it.ok = 1;
        it.g = __builtin_amdgcn_readfirstlane(u % a.groups);
        it.n = __builtin_amdgcn_readfirstlane(u / a.groups);
        it.oh0 = __builtin_amdgcn_readfirstlane(ti * TH);
        it.ow0 = __builtin_amdgcn_readfirstlane(tj * TW);
        return it;
    };
    // items of this workgroup: one, or (PERSIST) every gridDim.x-th id (gridDim.x is a multiple of 8)
    const int nitems = PERSIST ? __builtin_amdgcn_readfirstlane(((int)a.items - 1 - (int)blockIdx.x) / (int)gridDim.x + 1) : 1;
    auto item = [&](int j) __attribute__((always_inline)) -> Item {
        return j < nitems ? decode(blockIdx.x + j * gridDim.x) : Item{0, 0, 0, 0, 0, 0};
    };
    const Item it0 = item(0);
    if (!PERSIST && !it0.ok) return;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // tells the compiler it is wave-uniform
    const int wf = wave % WF, wp = wave / WF;
    const int li = lane & 15, kk = lane >> 4;

    const int plane = a.IH * a.IW;
    const T* const tnull = nullptr;
    const rsrc_t wrs = make_rsrc(a.wgt, a.wgt_bytes);

    // ---- per-thread gather plan for the source patch of an item (same for every chunk) ------------
    unsigned goff[XPT];  // byte offset inside the chunk's channels, kOob where the patch lies outside the image
    int loff[XPT];       // word offset inside a patch buffer
    const T* src = static_cast<const T*>(a.src);
    int xok = 0;
    auto plan_patch = [&](const Item& it) __attribute__((always_inline)) {
        xok = it.ok;
        src = static_cast<const T*>(a.src) + (size_t)(it.n * a.Csrc + it.g * a.Rg) * plane;
        const int ih0 = it.oh0 * ST - a.pad_h, iw0 = it.ow0 * ST - a.pad_w;
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            if constexpr (XW) {
                // 16-byte piece of the chunk's CK channels: TH full rows per channel, one contiguous run starting at
                // the tile's first row (the whole plane when the tile is the plane)
                const int f = tid + NT * m;
                const int c = (4 * f) / PSZ, rem = 4 * f - c * PSZ;
                goff[m] = f < XE / 4 ? (unsigned)(c * plane + it.oh0 * a.IW + rem) * 4u : kOob;
            } else {
                const int e = tid + NT * m;
                const int c = e / PSZ, rem = e - c * PSZ;
                const int ph = rem / PW, pw = rem - ph * PW;
                const int ih = ih0 + ph * GST, iw = iw0 + pw * GST;
                const bool ok = (e < XE) && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
                goff[m] = ok ? (unsigned)(c * plane + ih * a.IW + iw) * (unsigned)sizeof(T) : kOob;
            }
        }
    };
#pragma unroll
    for (int m = 0; m < XPT; ++m) {
        if constexpr (XW) {
            const int f = tid + NT * m;
            const int c = (4 * f) / PSZ, rem = 4 * f - c * PSZ;
            loff[m] = f < XE / 4 ? c * CS + rem : TRASH + (lane & ~3);   // 8-byte aligned: CS is even, rem a multiple of 4
        } else {
            const int e = tid + NT * m;
            const int c = e / PSZ, rem = e - c * PSZ;
            loff[m] = (e < XE) ? c * CS + rem : TRASH + lane;
        }
    }

    // ---- per-lane filter addressing of an item ----------------------------------------------
    // This wave's 16 filters; lane li owns filter f, lane group kk owns KQ consecutive channels.
    // forward:  w[(g*Fg+f)][c][tap]       -> contiguous over (c, tap) for a fixed filter
    // backward: w[(g*Rg+c)][f][RS-1-tap]  -> one run of RS values per reduction channel
    const int WRS = PHASE ? a.w_rs : RS;       // taps per (k, c) filter plane in memory
    const int wstep_k = BWD ? a.Fg * WRS : WRS;  // next reduction channel
    const int wstep_chunk = CK * wstep_k;      // next chunk
    // Byte offsets of the lane's KQ filter rows, kOob for an absent filter or channel.  Chunks are
    // visited in order, so the offsets of full chunks are running sums (one add each); only a
    // partial last chunk needs the per-channel test.
    unsigned wrun[KQ];
    bool f_ok = false;
    auto plan_filters = [&](const Item& it) __attribute__((always_inline)) {
        const int f = it.fblk * (16 * WF) + wf * 16 + li;
        f_ok = it.ok && f < a.Fg;
        const int wbase = BWD ? ((it.g * a.Rg + kk * KQ) * a.Fg + (f_ok ? f : 0)) * WRS
                              : ((it.g * a.Fg + (f_ok ? f : 0)) * a.Rg + kk * KQ) * WRS;
#pragma unroll
        for (int k4 = 0; k4 < KQ; ++k4) wrun[k4] = f_ok ? (unsigned)(wbase + k4 * wstep_k) * (unsigned)sizeof(T) : kOob;
    };

    // ---- per-lane pixel offsets into the LDS patch -----------------------------------------
    int pixoff[NBW];
    const bool quad_here = QUAD && wp == 0;                       // wave-uniform
    const bool last_ok = wp + WP * (NBWF - 1) < NBF;              // does this wave own a block in the last full slot?
    // block of slot i, and whether this wave owns it
    auto block_of = [&](int i) __attribute__((always_inline)) { return QUAD && i == NBW - 1 ? NB - 1 : wp + WP * i; };
    auto owns = [&](int i) __attribute__((always_inline)) {
        return QUAD && i == NBW - 1 ? (WP == 1 || quad_here) : !(NBF % WP != 0 && i == NBWF - 1 && !last_ok);
    };
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        int j = 16 * block_of(i) + (QUAD && i == NBW - 1 ? li & 3 : li);
        if (j >= NPX) j = 0;  // padding lanes read a valid address; their results are never stored
        const int th = j / TW, tw = j - th * TW;
        pixoff[i] = kk * KQ * CS + th * PST * PW + tw * PST;
    }

    // Per-tap LDS offset and accumulator set.  Plain correlation: tap (r, s) reads patch row r, column s.
    // MERGE2: tap index r reads patch row roff(r) = (r == 0) and belongs to row phase a = r % 2.
    constexpr auto tap_off = [](int t) {
        return MERGE2 ? ((t / S) == 0 ? PW : 0) + ((t % S) == 0 ? 1 : 0) : (t / S) * PW + (t % S);
    };
    constexpr auto tap_set = [](int t) { return MERGE2 ? ((t / S) % 2) * 2 + (t % S) % 2 : 0; };
    constexpr int NSET = MERGE2 ? 4 : 1;
    v4f acc[NSET][NBW];
#pragma unroll
    for (int q = 0; q < NSET; ++q)
#pragma unroll
        for (int i = 0; i < NBW; ++i) acc[q][i] = v4f{0.f, 0.f, 0.f, 0.f};

    float xreg[XW ? 1 : XPT];
    v4u xreg4[XW ? XPT : 1];

    // ---- fetching a chunk -------------------------------------------------------------------------
    // The patch descriptor covers exactly the channels the chunk still has, so a partial last chunk
    // (or a chunk past the end: zero channels) reads zeros without any per-element test.  The fetch
    // is cut into single load instructions ("pieces") so that the MFMA loop can issue them a few at
    // a time: issued in one burst they back up in the address unit and stall every wave.
    constexpr bool W4 = WV && !BWD && sizeof(T) == 4 && (RS * KQ) % 4 == 0;   // 4 filter values per load
    constexpr bool W3 = !W4 && !PHASE && sizeof(T) == 4 && RS % 3 == 0;       // 3 filter values per load
    constexpr int WPIECES = W4 ? RS * KQ / 4 : (W3 ? RS * KQ / 3 : RS * KQ);
    // Descriptor of chunk ch's patch: it covers exactly the channels the chunk has, so a partial last
    // chunk (or a chunk past the end: zero channels) reads zeros without any per-element test.
    auto patch_rsrc = [&](int ch) __attribute__((always_inline)) -> rsrc_t {
        const int left = xok ? a.Rg - ch * CK : 0;  // reduction channels from this chunk on (<= 0: no such chunk)
        const int have = left <= 0 ? 0 : (left < CK ? left : CK);
        return make_rsrc(src + (size_t)ch * CK * plane,
                         (unsigned)__builtin_amdgcn_readfirstlane(have * plane) * (unsigned)sizeof(T));
    };
    auto filter_offsets = [&](int ch, unsigned (&wvo)[KQ]) __attribute__((always_inline)) {
        const int left = a.Rg - ch * CK;
        if (left >= CK) {
#pragma unroll
            for (int k4 = 0; k4 < KQ; ++k4) wvo[k4] = wrun[k4];
        } else {
#pragma unroll
            for (int k4 = 0; k4 < KQ; ++k4) wvo[k4] = kk * KQ + k4 < left ? wrun[k4] : kOob;
        }
        // an absent filter stays out of range: kOob plus the whole tensor is still below 2^32
#pragma unroll
        for (int k4 = 0; k4 < KQ; ++k4) wrun[k4] += (unsigned)wstep_chunk * (unsigned)sizeof(T);
    };
    auto load_piece = [&](int piece, const rsrc_t& xrs) __attribute__((always_inline)) {
        if constexpr (XW) return __builtin_amdgcn_raw_buffer_load_b128(xrs, goff[piece], 0, 0);
        else return buf_load(xrs, goff[piece], tnull);
    };
    auto store_piece = [&](auto v, float* dst) __attribute__((always_inline)) {
        if constexpr (XW) {
            *reinterpret_cast<float2*>(dst) = make_float2(__uint_as_float(v[0]), __uint_as_float(v[1]));
            *reinterpret_cast<float2*>(dst + 2) = make_float2(__uint_as_float(v[2]), __uint_as_float(v[3]));
        } else {
            *dst = v;
        }
    };
    auto issue_x = [&](int piece, const rsrc_t& xrs) __attribute__((always_inline)) {
        if constexpr (XW) xreg4[piece] = load_piece(piece, xrs);
        else xreg[piece] = load_piece(piece, xrs);
    };
    auto store_x = [&](int piece, float* dst) __attribute__((always_inline)) {
        if constexpr (XW) store_piece(xreg4[piece], dst);
        else store_piece(xreg[piece], dst);
    };
    auto issue_w = [&](int q, const unsigned (&wvo)[KQ], float (&an)[RS * KQ]) __attribute__((always_inline)) {
        if constexpr (W4) {
            // forward: the lane's KQ channels x RS taps are RS*KQ consecutive floats (Rg is a multiple
            // of KQ, so they are all present or all absent)
            const v4u v = __builtin_amdgcn_raw_buffer_load_b128(wrs, wvo[0] + 16u * q, 0, 0);
            an[4 * q + 0] = __uint_as_float(v.x);
            an[4 * q + 1] = __uint_as_float(v.y);
            an[4 * q + 2] = __uint_as_float(v.z);
            an[4 * q + 3] = __uint_as_float(v.w);
        } else if constexpr (W3) {
            const int k4 = q / (RS / 3), j = q % (RS / 3);
            const v3u v = __builtin_amdgcn_raw_buffer_load_b96(wrs, wvo[k4] + 12u * j, 0, 0);
#pragma unroll
            for (int e = 0; e < 3; ++e) {
                const int t = 3 * j + e;   // tap as stored; backward-data uses it rotated by 180 degrees
                an[k4 * RS + (BWD && !MERGE2 ? RS - 1 - t : t)] = __uint_as_float(v[e]);
            }
        } else {
            const int k4 = q / RS, t = q % RS;
            if constexpr (PHASE)   // the table already lists the taps in correlation order
                an[k4 * RS + t] = buf_load(wrs, wvo[k4] + (unsigned)(a.tapoff[t] * sizeof(T)), tnull);
            else
                an[k4 * RS + (BWD && !MERGE2 ? RS - 1 - t : t)] = buf_load(wrs, wvo[k4] + (unsigned)(t * sizeof(T)), tnull);
        }
    };

    // One "group" = one (tap, reduction channel) pair = NBW MFMAs sharing an A operand; a chunk is G
    // groups.  Slot i of group g: the LDS read of operand i of group g+1, then MFMA i of group g (the
    // read issues while the matrix pipe is busy, every operand is requested a full group before its
    // use and, being issued first, is not given a register the MFMA still reads), then this slot's
    // share of the patch stores.
    constexpr int G = RS * KQ;
    static_assert(G >= 2, "a chunk needs a group for the stores and one for the loads");
    constexpr int SG = G >= 3 ? G / 3 : 1;      // groups that carry the patch stores
    constexpr int LG = G >= 3 ? G / 3 : 1;      // groups (after those) that carry the patch loads
    constexpr int WG = G >= 2 ? G / 2 : 1;      // groups that carry the filter loads
    constexpr int D = NBUF - 1;                 // the patch stored during chunk i belongs to chunk i + D
    float bq[2][NBW];
    // ac: filters of this chunk; an: register set the next chunk's filters are loaded into.
    // rd: this chunk's patch buffer; nx: the next chunk's; wr: the buffer stored to (word offsets in xs).
    // PAR: which half of bq holds group 0's operands (the halves alternate with the groups).
    // xch, wch: the chunks whose patch / filters are fetched during this one.
    auto compute = [&](auto parc, int xch, int wch, const float (&ac)[RS * KQ], float (&an)[RS * KQ], int rd, int nx, int wr)
                       __attribute__((always_inline)) {
        constexpr int PAR = decltype(parc)::value;
        // All loads in flight were issued at least a third of a chunk ago: the patch held in xreg and
        // this chunk's filters.  Retiring them here keeps waits on loads out of the loop.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        const rsrc_t xrs = patch_rsrc(xch);
        unsigned wvo[KQ];
        filter_offsets(wch, wvo);
        const float* pr[NBW];     // per-block read bases in this chunk's buffer
        const float* pn[NBW];     // ... and in the next chunk's
        float* ps[XPT];           // store addresses
#pragma unroll
        for (int i = 0; i < NBW; ++i) { pr[i] = xs + rd + pixoff[i]; pn[i] = xs + nx + pixoff[i]; }
#pragma unroll
        for (int m = 0; m < XPT; ++m) ps[m] = xs + wr + loff[m];
        if (NBUF == 2) {   // the buffer was completed by the barrier just passed: group 0's operands cannot be requested earlier
#pragma unroll
            for (int i = 0; i < NBW; ++i) bq[PAR][i] = pr[i][tap_off(0)];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int q = 0; q < WPIECES; ++q)
                if (q * WG / WPIECES == g) issue_w(q, wvo, an);
#pragma unroll
            for (int m = 0; m < XPT; ++m)
                if (SG + m * LG / XPT == g) issue_x(m, xrs);   // behind the store of the same register
            __builtin_amdgcn_sched_barrier(0);
            const int k4n = (g + 1) % KQ, tn = (g + 1) / KQ;
            const int off = k4n * CS + tap_off(tn);
            const float av = ac[(g % KQ) * RS + g / KQ];
#pragma unroll
            for (int i = 0; i < NBW; ++i) {
                const bool mine = owns(i);   // wave-uniform: this wave may have one block fewer
                if (mine) {
                    if (g + 1 < G) bq[(PAR + g + 1) & 1][i] = pr[i][off];
                    else if (NBUF == 3) bq[(PAR + g + 1) & 1][i] = pn[i][tap_off(0)];      // group 0 of the next chunk
                    if (QUAD && i == NBW - 1)
                        acc[tap_set(g / KQ)][i] = __builtin_amdgcn_mfma_f32_4x4x1f32(av, bq[(PAR + g) & 1][i], acc[tap_set(g / KQ)][i], 0, 0, 0);
                    else
                        acc[tap_set(g / KQ)][i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bq[(PAR + g) & 1][i], acc[tap_set(g / KQ)][i], 0, 0, 0);
                }
                {   // patch stores m with floor(m * SG*NBW / XPT) == this slot
                    constexpr int SACT = SG * NBW;
                    const int act = g * NBW + i;
                    const int lo = (act * XPT + SACT - 1) / SACT, hi = ((act + 1) * XPT + SACT - 1) / SACT;
#pragma unroll
                    for (int d = 0; d < (XPT + SACT - 1) / SACT + 1; ++d)
                        if (act < SACT && lo + d < hi && lo + d < XPT) store_x(lo + d, ps[lo + d]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // ---- write-out of an item: D[f = 4*kk+v][pixel = li] ---------------------------------------
    auto write_out = [&](const Item& it) __attribute__((always_inline)) {
        if (QUAD && quad_here) {
            // 4 x 4 x 1 blocks: lane 4 * (4 * kq + fg) + p holds in register v the partial sum over lane group kq's
            // channels for (filter 4 * fg + v, pixel p).  The 16 x 16 layout wants (filter 4 * kk + v, pixel li) in
            // lane 16 * kk + li: it adds the four partial sums of lanes p + 4 * kk + 16 * kq, kq in order.
#pragma unroll
            for (int q = 0; q < NSET; ++q)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float part = acc[q][NBW - 1][v];
                    float s = __shfl(part, (li & 3) + 4 * kk, 64);
#pragma unroll
                    for (int kq = 1; kq < 4; ++kq) s += __shfl(part, (li & 3) + 4 * kk + 16 * kq, 64);
                    acc[q][NBW - 1][v] = s;
                }
        }
        const int fq = it.fblk * (16 * WF) + wf * 16 + 4 * kk;
        const int dplane = PHASE || MERGE2 ? a.DH * a.DW : a.OH * a.OW;
        float* dst = a.dst + (size_t)(it.n * a.Cdst + it.g * a.Fg) * dplane;
        // Where accumulator set q of pixel block i goes: destination pixel index inside a plane, or -1 for none.
        // MERGE2: set (a, b) holds destination pixel (2*oh + 1 - a, 2*ow + 1 - b).
        auto pixel = [&](int i, int q, int& oh, int& ow) __attribute__((always_inline)) -> int {
            const int j = 16 * block_of(i) + li;
            const int th = j / TW, tw = j - th * TW;
            oh = it.oh0 + th; ow = it.ow0 + tw;
            if (!it.ok || !owns(i) || j >= NPX || oh >= a.OH || ow >= a.OW) return -1;
            const int dh = 2 * oh + 1 - q / 2, dw = 2 * ow + 1 - q % 2;
            if (MERGE2 && (dh >= a.DH || dw >= a.DW)) return -1;
            return MERGE2 ? dh * a.DW + dw : (PHASE ? (oh * a.o_sh + a.o_oh) * a.DW + ow * a.o_sw + a.o_ow : oh * a.OW + ow);
        };
        // Epilogues (wave-uniform branches on kernel arguments).  Bias + ReLU: the bias of the lane's four filters.
        if (a.bias) {
            float bv[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (it.ok && fq + v < a.Fg) bv[v] = a.bias[it.g * a.Fg + fq + v];
#pragma unroll
            for (int q = 0; q < NSET; ++q)
#pragma unroll
                for (int i = 0; i < NBW; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[q][i][v] = fmaxf(acc[q][i][v] + bv[v], 0.f);
        }
        // ReLU mask: the mask element under every result is requested first (buffer loads without branches, an
        // out-of-range offset where there is no result), so that the item waits for memory once, not per element.
        if (a.mask) {
            const rsrc_t mrs = make_rsrc(static_cast<const T*>(a.mask) + (size_t)(it.n * a.Cdst + it.g * a.Fg) * dplane,
                                         it.ok ? (unsigned)((size_t)a.Fg * dplane * sizeof(T)) : 0u);
            float mv[NSET][NBW][4];
#pragma unroll
            for (int q = 0; q < NSET; ++q)
#pragma unroll
                for (int i = 0; i < NBW; ++i) {
                    int oh, ow;
                    const int pix = pixel(i, q, oh, ow);
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        mv[q][i][v] = buf_load(mrs, pix >= 0 && fq + v < a.Fg ? (unsigned)((fq + v) * dplane + pix) * (unsigned)sizeof(T) : kOob, tnull);
                }
#pragma unroll
            for (int q = 0; q < NSET; ++q)
#pragma unroll
                for (int i = 0; i < NBW; ++i)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[q][i][v] = mv[q][i][v] > 0.f ? acc[q][i][v] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < NBW; ++i) {
#pragma unroll
            for (int q = 0; q < NSET; ++q) {
                int oh, ow;
                const int pix = pixel(i, q, oh, ow);
                if (pix < 0) continue;
                if (PHASE && a.fill2) {
                    // pix = (2 oh, 2 ow): the 2 x 2 block it heads belongs to this lane alone (no tap reaches the other three)
                    const bool right = 2 * ow + 1 < a.DW, below = 2 * oh + 1 < a.DH;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        if (fq + v >= a.Fg) continue;
                        float* o = dst + (size_t)(fq + v) * dplane + pix;
                        if (right && a.fill2 == 2) {   // even row length and aligned dx: 8-byte stores
                            *reinterpret_cast<float2*>(o) = make_float2(acc[q][i][v], 0.f);
                            if (below) *reinterpret_cast<float2*>(o + a.DW) = make_float2(0.f, 0.f);
                        } else {
                            o[0] = acc[q][i][v];
                            if (right) o[1] = 0.f;
                            if (below) o[a.DW] = 0.f;
                            if (below && right) o[a.DW + 1] = 0.f;
                        }
                    }
                    continue;
                }
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (fq + v < a.Fg) dst[(size_t)(fq + v) * dplane + pix] = acc[q][i][v];
            }
        }
    };

    // Two register sets for the filters alternate, so the loop is written out for an even and an odd
    // chunk (no register copies); the LDS buffers rotate through word offsets.
    float A0[RS * KQ], A1[RS * KQ];
    const int nchunks = (a.Rg + CK - 1) / CK;
    // The three positions of the pipeline (item, chunk): patch loads run D+1 chunks ahead of the
    // MFMAs, filter loads one chunk ahead.  Without PERSIST there is one item and chunks past its end
    // read zeros.
    int xj = 0, xch = 0, wj = 0, wch = 0, cj = 0, cch = 0;
    auto advance_patch = [&]() __attribute__((always_inline)) {
        ++xch;
        if (PERSIST && xch == nchunks) { xch = 0; ++xj; plan_patch(item(xj)); }
    };
    auto advance_filters = [&]() __attribute__((always_inline)) {
        ++wch;
        if (PERSIST && wch == nchunks) { wch = 0; ++wj; plan_filters(item(wj)); }
    };
    plan_patch(it0);
    plan_filters(it0);
    {   // prologue: chunks 0 .. D-1 into their buffers, chunk D into the registers, filters of chunk 0
        unsigned wvo[KQ];
        filter_offsets(wch, wvo);
        advance_filters();
#pragma unroll
        for (int q = 0; q < WPIECES; ++q) issue_w(q, wvo, A0);
        // all of them are requested before the first one is waited for
        decltype(load_piece(0, patch_rsrc(0))) pre[D][XPT];
#pragma unroll
        for (int c = 0; c < D; ++c) {
            const rsrc_t xrs = patch_rsrc(xch);
#pragma unroll
            for (int m = 0; m < XPT; ++m) pre[c][m] = load_piece(m, xrs);
            advance_patch();
        }
        {
            const rsrc_t xrs = patch_rsrc(xch);
#pragma unroll
            for (int m = 0; m < XPT; ++m) issue_x(m, xrs);
            advance_patch();
        }
#pragma unroll
        for (int c = 0; c < D; ++c)
#pragma unroll
            for (int m = 0; m < XPT; ++m) store_piece(pre[c][m], xs + c * BUFSZ + loff[m]);
        __syncthreads();
        if (NBUF == 3) {
#pragma unroll
            for (int i = 0; i < NBW; ++i) bq[0][i] = xs[pixoff[i] + tap_off(0)];
        }
    }
    int rd = 0, nx = BUFSZ, wr = D * BUFSZ;
    // after a chunk: move the fetch positions on; an item whose last chunk this was is written out
    auto chunk_done = [&]() __attribute__((always_inline)) {
        advance_patch();
        advance_filters();
        if (PERSIST && ++cch == nchunks) {
            write_out(item(cj));
#pragma unroll
            for (int q = 0; q < NSET; ++q)
#pragma unroll
                for (int i = 0; i < NBW; ++i) acc[q][i] = v4f{0.f, 0.f, 0.f, 0.f};
            cch = 0;
            ++cj;
        }
        __syncthreads();
        rd = nx;
        nx = nx + BUFSZ == NBUF * BUFSZ ? 0 : nx + BUFSZ;
        wr = wr + BUFSZ == NBUF * BUFSZ ? 0 : wr + BUFSZ;
    };
    const int total = nitems * nchunks;
    for (int ch = 0; ch < total; ch += 2) {
        compute(std::integral_constant<int, 0>{}, xch, wch, A0, A1, rd, nx, wr);
        chunk_done();
        if (ch + 1 >= total) break;
        compute(std::integral_constant<int, G & 1>{}, xch, wch, A1, A0, rd, nx, wr);
        chunk_done();
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // loads fetched past the last chunk still target registers
    if (!PERSIST) write_out(it0);
}


}  // namespace tile
}  // namespace miconv
