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
//   * Global loads for chunk i+1 are issued before the MFMA work of chunk i and
//     land in the other LDS buffer afterwards: one barrier per chunk.
#include "common.h"

namespace miconv {
namespace tile {

typedef float v4f __attribute__((ext_vector_type(4)));

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
};

// Buffer loads: the hardware compares the byte offset with the descriptor's size and returns 0
// beyond it, so an element that must read as zero (outside the image, past the last channel, an
// absent filter) is given the offset kOob and costs neither a branch nor a select on the result.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v3u __attribute__((ext_vector_type(3)));
constexpr unsigned kOob = 0x80000000u;  // tensors handled here are smaller than 2 GiB
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const float*) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0));
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const uint16_t*) {
    return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_raw_buffer_load_b16(r, byte_off, 0, 0)) << 16);
}

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
template <typename T, int R, int S, int ST, int TH, int TW, int CK, int WF, int WP, bool BWD, bool WV, bool PHASE>
__global__ __launch_bounds__(64 * WF * WP) void conv_tile_kernel(TileArgs a) {
    constexpr int NT = 64 * WF * WP;
    constexpr int RS = R * S;
    constexpr int PH = (TH - 1) * ST + R, PW = (TW - 1) * ST + S;
    constexpr int PSZ = PH * PW;
    constexpr int KQ = CK / 4;  // channels per lane group: lane group kk owns channels [kk*KQ, kk*KQ+KQ) of a chunk
    static_assert(CK == 4 || CK == 8 || CK == 16 || CK == 32, "CK must be 4, 8, 16 or 32");
    constexpr int CS = lds_channel_stride(PSZ, KQ);
    constexpr int XE = CK * PSZ;
    constexpr int XPT = (XE + NT - 1) / NT;
    constexpr int NPX = TH * TW;
    constexpr int NB = (NPX + 15) / 16;      // 16-pixel blocks in the tile
    constexpr int NBW = (NB + WP - 1) / WP;  // blocks per wave

    __shared__ float xs[2][CK * CS];

    // ---- which unit of work -------------------------------------------------------------
    // Consecutive workgroup ids land on different XCDs (8 of them, one L2 each).  All filter
    // blocks of one (image, tile) are given ids that differ by multiples of 8 so that they share an L2.
    const int b = blockIdx.x;
    const int xcd = b & 7;
    const int rest = b >> 3;
    const int fblk = rest % a.fblocks;
    const int unit = (rest / a.fblocks) * 8 + xcd;
    if (unit >= a.units) return;
    int u = unit;
    const int tj = u % a.tiles_w; u /= a.tiles_w;
    const int ti = u % a.tiles_h; u /= a.tiles_h;
    const int g = u % a.groups;
    const int n = u / a.groups;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // tells the compiler it is wave-uniform
    const int wf = wave % WF, wp = wave / WF;
    const int li = lane & 15, kk = lane >> 4;

    const int oh0 = ti * TH, ow0 = tj * TW;
    const int ih0 = oh0 * ST - a.pad_h, iw0 = ow0 * ST - a.pad_w;
    const int plane = a.IH * a.IW;

    const T* src = static_cast<const T*>(a.src) + (size_t)(n * a.Csrc + g * a.Rg) * plane;
    const T* const tnull = nullptr;
    const rsrc_t wrs = make_rsrc(a.wgt, a.wgt_bytes);

    // ---- per-thread gather plan for the source patch (same for every chunk) ---------------
    unsigned goff[XPT];  // byte offset inside the chunk's channels, kOob where the patch lies outside the image
    int loff[XPT];
#pragma unroll
    for (int m = 0; m < XPT; ++m) {
        const int e = tid + NT * m;
        const int c = e / PSZ, rem = e - c * PSZ;
        const int ph = rem / PW, pw = rem - ph * PW;
        const int ih = ih0 + ph, iw = iw0 + pw;
        const bool ok = (e < XE) && ih >= 0 && ih < a.IH && iw >= 0 && iw < a.IW;
        goff[m] = ok ? (unsigned)(c * plane + ih * a.IW + iw) * (unsigned)sizeof(T) : kOob;
        loff[m] = (e < XE) ? c * CS + rem : -1;
    }

    // ---- per-lane filter addressing ---------------------------------------------------------
    // This wave's 16 filters; lane li owns filter f, lane group kk owns KQ consecutive channels.
    const int f = fblk * (16 * WF) + wf * 16 + li;
    const bool f_ok = f < a.Fg;
    // forward:  w[(g*Fg+f)][c][tap]       -> contiguous over (c, tap) for a fixed filter
    // backward: w[(g*Rg+c)][f][RS-1-tap]  -> one run of RS values per reduction channel
    const int WRS = PHASE ? a.w_rs : RS;       // taps per (k, c) filter plane in memory
    const int wbase = BWD ? ((g * a.Rg + kk * KQ) * a.Fg + (f_ok ? f : 0)) * WRS
                          : ((g * a.Fg + (f_ok ? f : 0)) * a.Rg + kk * KQ) * WRS;
    const int wstep_k = BWD ? a.Fg * WRS : WRS;  // next reduction channel
    const int wstep_chunk = CK * wstep_k;      // next chunk

    // ---- per-lane pixel offsets into the LDS patch -----------------------------------------
    int pixoff[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        int j = 16 * (wp + WP * i) + li;
        if (j >= NPX) j = 0;  // padding lanes read a valid address; their results are never stored
        const int th = j / TW, tw = j - th * TW;
        pixoff[i] = kk * KQ * CS + th * ST * PW + tw * ST;
    }

    const bool last_ok = wp + WP * (NBW - 1) < NB;   // does this wave own a block in its last slot?
    v4f acc[NBW];
#pragma unroll
    for (int i = 0; i < NBW; ++i) acc[i] = v4f{0.f, 0.f, 0.f, 0.f};

    float xreg[XPT];

    // ---- fetching a chunk -------------------------------------------------------------------------
    // The patch descriptor covers exactly the channels the chunk still has, so a partial last chunk
    // (or a chunk past the end: zero channels) reads zeros without any per-element test.  The fetch
    // is cut into single load instructions ("pieces") so that the MFMA loop can issue them a few at
    // a time: issued in one burst they back up in the address unit and stall every wave.
    constexpr bool W4 = WV && !BWD && sizeof(T) == 4 && (RS * KQ) % 4 == 0;   // 4 filter values per load
    constexpr bool W3 = !W4 && !PHASE && sizeof(T) == 4 && RS % 3 == 0;       // 3 filter values per load
    constexpr int WPIECES = W4 ? RS * KQ / 4 : (W3 ? RS * KQ / 3 : RS * KQ);
    constexpr int NPIECES = XPT + WPIECES;
    auto prepare = [&](int ch, rsrc_t& xrs, unsigned (&wvo)[KQ]) {
        const int left = a.Rg - ch * CK;  // reduction channels from this chunk on (<= 0: no such chunk)
        const int have = left <= 0 ? 0 : (left < CK ? left : CK);
        xrs = make_rsrc(src + (size_t)ch * CK * plane,
                        (unsigned)__builtin_amdgcn_readfirstlane(have * plane) * (unsigned)sizeof(T));
        const int wb = wbase + ch * wstep_chunk;
#pragma unroll
        for (int k4 = 0; k4 < KQ; ++k4)
            wvo[k4] = (f_ok && kk * KQ + k4 < left) ? (unsigned)(wb + k4 * wstep_k) * (unsigned)sizeof(T) : kOob;
    };
    auto issue = [&](int piece, const rsrc_t& xrs, const unsigned (&wvo)[KQ], float (&an)[RS * KQ]) {
        if (piece < XPT) {
            xreg[piece] = buf_load(xrs, goff[piece], tnull);
            return;
        }
        const int q = piece - XPT;
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
                an[k4 * RS + (BWD ? RS - 1 - t : t)] = __uint_as_float(v[e]);
            }
        } else {
            const int k4 = q / RS, t = q % RS;
            if constexpr (PHASE)   // the table already lists the taps in correlation order
                an[k4 * RS + t] = buf_load(wrs, wvo[k4] + (unsigned)(a.tapoff[t] * sizeof(T)), tnull);
            else
                an[k4 * RS + (BWD ? RS - 1 - t : t)] = buf_load(wrs, wvo[k4] + (unsigned)(t * sizeof(T)), tnull);
        }
    };
    auto store_patch = [&](float* buf) {
        // Everything fetched for the next chunk (patch and filters) was issued during the MFMA loop;
        // retiring all of it here keeps waits on these loads out of the next MFMA loop.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
#pragma unroll
        for (int m = 0; m < XPT; ++m)
            if (loff[m] >= 0) buf[loff[m]] = xreg[m];
    };
    // One "group" = one (tap, reduction channel) pair = NBW MFMAs sharing an A operand.  While chunk i
    // is multiplied out of xb/ac, the pieces of chunk i+1 are issued into xreg/an.
    auto compute = [&](const float* xb, const float (&ac)[RS * KQ], const rsrc_t& xrs, const unsigned (&wvo)[KQ],
                       float (&an)[RS * KQ]) {
        constexpr int G = RS * KQ;
        // The next chunk's pieces all go out in the first half of the groups, so that the remaining MFMA
        // work covers their latency before store_patch() waits for them.
        constexpr int ISSUE_GROUPS = G >= 2 ? G / 2 : 1;
        float bq[2][NBW];
#pragma unroll
        for (int i = 0; i < NBW; ++i) bq[0][i] = xb[pixoff[i]];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int piece = 0; piece < NPIECES; ++piece)
                if (piece * ISSUE_GROUPS / NPIECES == g) issue(piece, xrs, wvo, an);
            __builtin_amdgcn_sched_barrier(0);
            const int k4n = (g + 1) % KQ, tn = (g + 1) / KQ;
            const int off = k4n * CS + (tn / S) * PW + (tn % S);
            const float av = ac[(g % KQ) * RS + g / KQ];
            // The LDS read of operand i of the next group, then MFMA i of this group: the read issues while
            // the matrix pipe is busy with MFMA i-1, every operand is requested a full group before its
            // use, and (being issued first) the read cannot be given a register the MFMA still reads.
#pragma unroll
            for (int i = 0; i < NBW; ++i) {
                if (NB % WP != 0 && i == NBW - 1 && !last_ok) continue;   // wave-uniform: this wave has one block fewer
                if (g + 1 < G) bq[(g + 1) & 1][i] = xb[pixoff[i] + off];
                acc[i] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, bq[g & 1][i], acc[i], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    // Two register sets for the filters and two LDS buffers for the patch alternate, so the loop
    // is written out for an even and an odd chunk: no register copies, LDS addresses are immediates.
    float A0[RS * KQ], A1[RS * KQ];
    const int nchunks = (a.Rg + CK - 1) / CK;
    rsrc_t xrs;
    unsigned wvo[KQ];
    prepare(0, xrs, wvo);
#pragma unroll
    for (int piece = 0; piece < NPIECES; ++piece) issue(piece, xrs, wvo, A0);
    store_patch(xs[0]);
    __syncthreads();
    for (int ch = 0; ch < nchunks; ch += 2) {
        prepare(ch + 1, xrs, wvo);
        compute(xs[0], A0, xrs, wvo, A1);
        if (ch + 1 >= nchunks) break;
        store_patch(xs[1]);
        __syncthreads();
        prepare(ch + 2, xrs, wvo);
        compute(xs[1], A1, xrs, wvo, A0);
        if (ch + 2 < nchunks) store_patch(xs[0]);
        __syncthreads();
    }

    // ---- epilogue: D[f = 4*kk+v][pixel = li] ---------------------------------------------------
    const int fq = fblk * (16 * WF) + wf * 16 + 4 * kk;
    const int dplane = PHASE ? a.DH * a.DW : a.OH * a.OW;
    float* dst = a.dst + (size_t)(n * a.Cdst + g * a.Fg) * dplane;
#pragma unroll
    for (int i = 0; i < NBW; ++i) {
        const int j = 16 * (wp + WP * i) + li;
        if (j >= NPX) continue;
        const int th = j / TW, tw = j - th * TW;
        const int oh = oh0 + th, ow = ow0 + tw;
        if (oh >= a.OH || ow >= a.OW) continue;
        const int pix = PHASE ? (oh * a.o_sh + a.o_oh) * a.DW + ow * a.o_sw + a.o_ow : oh * a.OW + ow;
#pragma unroll
        for (int v = 0; v < 4; ++v)
            if (fq + v < a.Fg) dst[(size_t)(fq + v) * dplane + pix] = acc[i][v];
    }
}


}  // namespace tile
}  // namespace miconv
