// Backward-weight convolution on the fp32 matrix cores (v_mfma_f32_16x16x4_f32), gfx950.
//
//   dw[k,c,r,s] = sum_{n,p,q} dy[n,k,p,q] * x[n, g*Cg+c, p*ST-pad_h+r, q*ST-pad_w+s]
//
// As a GEMM the output is Kg x (Cg*R*S) and the reduction runs over all N*P*Q
// output pixels.  MFMA roles: M = 16 output channels k (A from dy), N = 16 input
// channels c (B from x), K = 4 output pixels; one accumulator block per filter tap.
//
// Decomposition.  A workgroup owns 16*KB output channels x 16*CB input channels
// (all R*S taps) of one group and a contiguous share ("split") of the stages; a
// stage is one image and one TH x TW rectangle of output pixels.  Per stage the
// dy tile and the x patch under it (zero-filled outside the image) are gathered
// into LDS with coalesced row reads; the tap shift is an LDS address offset, so
// every x value is read from global memory once per stage and reused R*S times.
// Waves are arranged WK x WC x WS: WK and WC divide the accumulator blocks, WS
// divides the pixel steps of a stage.  Stage i+1 is fetched into registers while
// stage i is multiplied and is written to the other LDS buffer afterwards.
// At the end the WS partial accumulators are summed through LDS in a fixed order
// and written with coalesced stores, either to dw (one split) or to a partial
// buffer that reduce_splits_kernel sums in split order: no floating-point
// atomics anywhere, so dw is bit-reproducible.
#include "common.h"

namespace miconv {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));

struct WgradArgs {
    const void* x;
    const void* dy;
    float* out;        // dw, or the partial buffer [nsplit][K*Cg*R*S]
    int N, C, H, W, K, P, Q;
    int Cg, Kg, groups;
    int pad_h, pad_w;
    int tiles_h, tiles_w;
    int kblocks, cblocks;  // per group
    int nsplit, stages;    // stages = tiles_h*tiles_w*img_stages, ordered tile-major
    int img_stages;        // ceil(N / images per stage)
    int total_wgs;
    int xk, xc;            // blocks of one XCD form an xk x xc rectangle of the (k, c) block grid (0: linear runs)
};

// Buffer loads return 0 for a byte offset at or beyond the descriptor's size: elements that must
// read as zero (outside the image or the tile, absent channels) are given the offset kOob.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr unsigned kOob = 0x80000000u;  // one image's channels are far smaller than 2 GiB
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const float*) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0));
}
__device__ __forceinline__ float buf_load(rsrc_t r, unsigned byte_off, const uint16_t*) {
    return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_raw_buffer_load_b16(r, byte_off, 0, 0)) << 16);
}

constexpr int next_2_mod_4(int v) { return v + ((6 - v % 4) % 4); }   // smallest >= v that is 2 mod 4
constexpr int next_odd(int v) { return v | 1; }
constexpr int cmax(int a, int b) { return a > b ? a : b; }

// IMG: images per stage.  With 4 waves sharing the pixel steps of a stage, two 14x14 images (98 steps)
// divide almost evenly (25/25/24/24) where one (49 steps) leaves three waves idle for a step in 13.
// WIDE: the tile is the whole output plane and the planes are multiples of 4 floats: dy rows and x
// planes are then read as 16-byte pieces (a quarter of the address-unit work of 4-byte reads) and the
// x values scattered into the zero-bordered patch, whose border words are written once.
template <typename T, int R, int S, int ST, int TH, int TW, int KB, int CB, int WK, int WC, int WS, int IMG, bool WIDE>
__global__ __launch_bounds__(64 * WK * WC * WS) void wgrad_kernel(WgradArgs a) {
    constexpr int NT = 64 * WK * WC * WS;
    constexpr int RS = R * S;
    constexpr int PH = (TH - 1) * ST + R, PW = (TW - 1) * ST + S, PSZ = PH * PW;
    constexpr int NPX = TH * TW;
    static_assert(NPX % 4 == 0, "tile pixels must fill whole MFMA steps");
    static_assert(KB % WK == 0 && CB % WC == 0, "wave grid must divide the block grid");
    constexpr int SPI = NPX / 4;           // steps per image
    constexpr int NSTEPS = IMG * SPI;
    constexpr int KBW = KB / WK, CBW = CB / WC;
    // LDS row strides: 16 lanes x 2 adjacent pixels must fall in 32 distinct banks.
    constexpr int DS = next_2_mod_4(NPX);
    constexpr int XS = ST == 1 ? next_2_mod_4(PSZ) : next_odd(PSZ);
    constexpr int YE = 16 * KB * NPX, XE = 16 * CB * PSZ;               // per image
    constexpr int YPT = WIDE ? (IMG * YE / 4 + NT - 1) / NT : (IMG * YE + NT - 1) / NT;   // load pieces per thread
    constexpr int XPT = WIDE ? (IMG * 16 * CB * (NPX * ST * ST) / 4 + NT - 1) / NT : (IMG * XE + NT - 1) / NT;
    constexpr int YIMG = 16 * KB * DS, XIMG = 16 * CB * XS;             // floats per image in LDS
    constexpr int STAGE = IMG * (YIMG + XIMG);                          // floats per LDS buffer
    constexpr int OUTSZ = 16 * KB * 16 * CB * RS;                       // accumulator elements of the workgroup
    constexpr int LDSF = cmax(2 * STAGE, WS * OUTSZ);
    static_assert(LDSF * 4 <= 160 * 1024, "LDS budget");

    __shared__ float lds[LDSF];

    // ---- which output block / split ----------------------------------------------------------
    // Workgroup ids are dealt round-robin to the 8 XCDs; giving each XCD a contiguous run of
    // block ids makes the blocks that share dy tiles and x patches share an L2.
    // A rectangle of blocks reads xk dy tiles and xc x patches per stage, so the squarer it is the
    // less each L2 has to fetch from memory.
    int cbi, kbi, g, sp;
    if (a.xk > 0) {
        const int xcd = blockIdx.x & 7, l = blockIdx.x >> 3;   // l < xk * xc
        const int across = a.cblocks / a.xc;                   // XCD rectangles per row of the block grid
        kbi = (xcd / across) * a.xk + l / a.xc;
        cbi = (xcd % across) * a.xc + l % a.xc;
        g = 0; sp = 0;
    } else {
        const int per_xcd = (a.total_wgs + 7) / 8;
        const int L = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
        if (L >= a.total_wgs) return;
        int u = L;
        cbi = u % a.cblocks; u /= a.cblocks;
        kbi = u % a.kblocks; u /= a.kblocks;
        g = u % a.groups;
        sp = u / a.groups;
    }

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int li = lane & 15, kk = lane >> 4;
    const int wk = wave % WK, wc = (wave / WK) % WC, ws = wave / (WK * WC);

    const int k0 = kbi * 16 * KB, c0 = cbi * 16 * CB;   // within the group
    // a stage = IMG consecutive images of one tile; stages are ordered tile-major
    const int s_begin = (int)((long long)a.stages * sp / a.nsplit);
    const int s_end = (int)((long long)a.stages * (sp + 1) / a.nsplit);

    const T* xg = static_cast<const T*>(a.x);
    const T* dyg = static_cast<const T*>(a.dy);
    const int xplane = a.H * a.W, yplane = a.P * a.Q;
    const T* const tnull = nullptr;

    // ---- gather plans (depend on the tile position only) -----------------------------------------
    // Offsets are relative to the first image of the stage; image i of the stage adds i whole images.
    // Images past the end of the batch fall outside the descriptor and read as zero.
    unsigned ygo[YPT], xgo[XPT];   // byte offsets, kOob = reads as zero
    int ylo[WIDE ? YPT : 1], xlo[WIDE ? XPT : 1][4];   // wide path: where the pieces land in a stage's LDS buffer
    auto plan = [&](int tile) {
        if constexpr (WIDE) {
            // whole planes: H*W == NPX*ST*ST is not required, only that an x plane is xplane floats
            const int xq = xplane / 4;   // float4 per x plane
#pragma unroll
            for (int m = 0; m < YPT; ++m) {
                const int f = tid + NT * m;
                const int im = f / (YE / 4), ei = 4 * f - im * YE;
                const int kl = ei / NPX, px = ei - kl * NPX;
                const bool ok = f < IMG * YE / 4 && k0 + kl < a.Kg;
                ygo[m] = ok ? (unsigned)((im * a.K + g * a.Kg + k0 + kl) * yplane + px) * 4u : kOob;
                ylo[m] = f < IMG * YE / 4 ? im * YIMG + kl * DS + px : -1;
            }
#pragma unroll
            for (int m = 0; m < XPT; ++m) {
                const int f = tid + NT * m;
                const int pc = f / xq, rem = 4 * (f - pc * xq);      // plane (image-major, then channel), element
                const int im = pc / (16 * CB), cl = pc - im * 16 * CB;
                const bool ok = pc < IMG * 16 * CB && c0 + cl < a.Cg;
                xgo[m] = ok ? (unsigned)((im * a.C + g * a.Cg + c0 + cl) * xplane + rem) * 4u : kOob;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int ih = (rem + e) / a.W, iw = (rem + e) - ih * a.W;
                    const int ph = ih + a.pad_h, pw = iw + a.pad_w;
                    const bool in = pc < IMG * 16 * CB && ph >= 0 && ph < PH && pw >= 0 && pw < PW;
                    xlo[m][e] = in ? IMG * YIMG + im * XIMG + cl * XS + ph * PW + pw : -1;
                }
            }
            return;
        }
        const int ti = tile / a.tiles_w, tj = tile - ti * a.tiles_w;
        const int p0 = ti * TH, q0 = tj * TW;
        const int h0 = p0 * ST - a.pad_h, v0 = q0 * ST - a.pad_w;
#pragma unroll
        for (int m = 0; m < YPT; ++m) {
            const int e = tid + NT * m;
            const int im = e / YE, ei = e - im * YE;
            const int kl = ei / NPX, px = ei - kl * NPX;
            const int th = px / TW, tw = px - th * TW;
            const int p = p0 + th, q = q0 + tw;
            const bool ok = e < IMG * YE && k0 + kl < a.Kg && p < a.P && q < a.Q;
            ygo[m] = ok ? (unsigned)((im * a.K + g * a.Kg + k0 + kl) * yplane + p * a.Q + q) * (unsigned)sizeof(T) : kOob;
        }
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int e = tid + NT * m;
            const int im = e / XE, ei = e - im * XE;
            const int cl = ei / PSZ, rem = ei - cl * PSZ;
            const int ph = rem / PW, pw = rem - ph * PW;
            const int h = h0 + ph, v = v0 + pw;
            const bool ok = e < IMG * XE && c0 + cl < a.Cg && h >= 0 && h < a.H && v >= 0 && v < a.W;
            xgo[m] = ok ? (unsigned)((im * a.C + g * a.Cg + c0 + cl) * xplane + h * a.W + v) * (unsigned)sizeof(T) : kOob;
        }
    };

    // The fetch of a stage is cut into single load instructions ("pieces") that the MFMA loop issues
    // a few at a time; issued in one burst they back up in the address unit and stall every wave.
    float yreg[WIDE ? 1 : YPT], xreg[WIDE ? 1 : XPT];
    v4u yreg4[WIDE ? YPT : 1], xreg4[WIDE ? XPT : 1];
    constexpr int NPIECES = YPT + XPT;
    auto descriptors = [&](int stage, rsrc_t& yrs, rsrc_t& xrs) {
        const int n = (stage % a.img_stages) * IMG;          // first image of the stage
        const int left = stage < s_end ? a.N - n : 0;        // images from here to the end of the batch
        const int have = left < IMG ? left : IMG;
        yrs = make_rsrc(dyg + (size_t)n * a.K * yplane, (unsigned)(have * a.K * yplane) * (unsigned)sizeof(T));
        xrs = make_rsrc(xg + (size_t)n * a.C * xplane, (unsigned)(have * a.C * xplane) * (unsigned)sizeof(T));
    };
    auto issue = [&](int piece, const rsrc_t& yrs, const rsrc_t& xrs) {
        if constexpr (WIDE) {
            if (piece < YPT) yreg4[piece] = __builtin_amdgcn_raw_buffer_load_b128(yrs, ygo[piece], 0, 0);
            else xreg4[piece - YPT] = __builtin_amdgcn_raw_buffer_load_b128(xrs, xgo[piece - YPT], 0, 0);
        } else {
            if (piece < YPT) yreg[piece] = buf_load(yrs, ygo[piece], tnull);
            else xreg[piece - YPT] = buf_load(xrs, xgo[piece - YPT], tnull);
        }
    };
    auto stash = [&](int buf) {
        // Everything fetched for the next stage was issued during the MFMA loop; retiring all of it
        // here keeps waits on these loads out of the next MFMA loop.
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
        float* sb = lds + buf * STAGE;
        if constexpr (WIDE) {
#pragma unroll
            for (int m = 0; m < YPT; ++m)
                if (ylo[m] >= 0) {   // rows are 8-byte aligned in LDS (DS is even, px a multiple of 4)
                    *reinterpret_cast<float2*>(sb + ylo[m]) = make_float2(__uint_as_float(yreg4[m].x), __uint_as_float(yreg4[m].y));
                    *reinterpret_cast<float2*>(sb + ylo[m] + 2) = make_float2(__uint_as_float(yreg4[m].z), __uint_as_float(yreg4[m].w));
                }
#pragma unroll
            for (int m = 0; m < XPT; ++m)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (xlo[m][e] >= 0) sb[xlo[m][e]] = __uint_as_float(xreg4[m][e]);
            return;
        }
#pragma unroll
        for (int m = 0; m < YPT; ++m) {
            const int e = tid + NT * m;
            const int im = e / YE, ei = e - im * YE;
            const int kl = ei / NPX, px = ei - kl * NPX;
            if (e < IMG * YE) sb[im * YIMG + kl * DS + px] = yreg[m];
        }
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int e = tid + NT * m;
            const int im = e / XE, ei = e - im * XE;
            const int cl = ei / PSZ, rem = ei - cl * PSZ;
            if (e < IMG * XE) sb[IMG * YIMG + im * XIMG + cl * XS + rem] = xreg[m];
        }
    };

    v4f acc[KBW][CBW][RS];
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int j = 0; j < CBW; ++j)
#pragma unroll
            for (int t = 0; t < RS; ++t) acc[i][j][t] = v4f{0.f, 0.f, 0.f, 0.f};

    // ---- this wave's pixel steps: t = ws, ws+WS, ...; the LDS offsets of its lanes never change ----
    constexpr int IT_FULL = NSTEPS / WS, IT_REM = NSTEPS % WS, ITER = IT_FULL + (IT_REM ? 1 : 0);
    int yoff[ITER], xoff[ITER];
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
        int t = ws + WS * i;
        if (t >= NSTEPS) t = NSTEPS - 1;   // only in the step that waves with ws >= IT_REM skip; keeps the read in range
        const int im = t / SPI;
        const int px = 4 * (t - im * SPI) + kk;
        const int th = px / TW, tw = px - th * TW;
        yoff[i] = im * YIMG + (16 * (wk * KBW) + li) * DS + px;
        xoff[i] = IMG * YIMG + im * XIMG + (16 * (wc * CBW) + li) * XS + th * ST * PW + tw * ST;
    }

    // One step = NM = KBW*CBW*RS MFMAs on NR = KBW + CBW*RS operands.  Operand r of step i+1 is read
    // from LDS right before MFMA r of step i, so reads issue while the matrix pipe is busy and every
    // operand is requested a full step before its use; scheduling fences pin that order.
    constexpr int NM = KBW * CBW * RS, NR = KBW + CBW * RS;
    // The next stage's pieces all go out in the first third of the steps, so that the rest of the
    // stage's MFMA work covers their latency before stash() waits for them.
    constexpr int ISSUE_STEPS = ITER >= 3 ? ITER / 3 : 1;
    auto multiply = [&](const float* sb, const rsrc_t& yrs, const rsrc_t& xrs) {
        float ops[2][NR];   // [0..KBW): dy operands, then CBW*RS x operands
        auto read_op = [&](int i, int r) -> float {
            if (r < KBW) return sb[yoff[i] + r * 16 * DS];
            const int q = r - KBW, j = q / RS, t = q % RS;
            return sb[xoff[i] + j * 16 * XS + (t / S) * PW + (t % S)];
        };
#pragma unroll
        for (int r = 0; r < NR; ++r) ops[0][r] = read_op(0, r);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < ITER; ++i) {
#pragma unroll
            for (int piece = 0; piece < NPIECES; ++piece)
                if (piece * ISSUE_STEPS / NPIECES == i) issue(piece, yrs, xrs);
            __builtin_amdgcn_sched_barrier(0);
            const bool next = i + 1 < ITER;
            if (i < IT_FULL || ws < IT_REM) {  // wave-uniform; false only in the last step
#pragma unroll
                for (int m = 0; m < (NM > NR ? NM : NR); ++m) {
                    // The read goes first: the register it fills must differ from the ones the MFMA
                    // behind it still reads (a read that overwrote an operand of the MFMA just issued
                    // would have to wait for that MFMA to fetch it).
                    if (next && m < NR) ops[(i + 1) & 1][m] = read_op(i + 1, m);
                    if (m < NM) {
                        const int j = m / (RS * KBW), t = (m / KBW) % RS, ib = m % KBW;
                        acc[ib][j][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ops[i & 1][ib], ops[i & 1][KBW + j * RS + t],
                                                                             acc[ib][j][t], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    if constexpr (WIDE) {
        // patch borders (and everything else) start as zero; the scatter only writes interior words
        for (int e = tid; e < 2 * STAGE; e += NT) lds[e] = 0.f;
        __syncthreads();
    }
    if (s_begin < s_end) {
        int tile = s_begin / a.img_stages;
        plan(tile);
        rsrc_t yrs, xrs;
        descriptors(s_begin, yrs, xrs);
#pragma unroll
        for (int piece = 0; piece < NPIECES; ++piece) issue(piece, yrs, xrs);
        stash(0);
        __syncthreads();
        int buf = 0;
        for (int stage = s_begin; stage < s_end; ++stage) {
            const bool more = stage + 1 < s_end;
            if (more) {
                const int nt = (stage + 1) / a.img_stages;
                if (nt != tile) { tile = nt; plan(tile); }
            }
            descriptors(stage + 1, yrs, xrs);   // past the split's end: empty descriptors, every load reads zero
            multiply(lds + buf * STAGE, yrs, xrs);
            if (more) stash(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    // ---- combine the WS pixel-step shares and write out ---------------------------------------------
    // LDS layout of one share: [k local][c local][tap], i.e. the order of dw within the block.
    __syncthreads();
    constexpr int ROW = 16 * CB * RS;
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int j = 0; j < CBW; ++j)
#pragma unroll
            for (int t = 0; t < RS; ++t)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int kl = 16 * (wk * KBW + i) + 4 * kk + v;
                    const int cl = 16 * (wc * CBW + j) + li;
                    lds[ws * OUTSZ + kl * ROW + cl * RS + t] = acc[i][j][t][v];
                }
    __syncthreads();
    const size_t wsize = (size_t)a.K * a.Cg * RS;
    float* out = a.out + (a.nsplit > 1 ? (size_t)sp * wsize : 0);
    for (int o = tid; o < OUTSZ; o += NT) {
        const int kl = o / ROW, rem = o - kl * ROW;
        const int cl = rem / RS;
        if (k0 + kl >= a.Kg || c0 + cl >= a.Cg) continue;
        float sum = lds[o];
#pragma unroll
        for (int w = 1; w < WS; ++w) sum += lds[w * OUTSZ + o];
        out[((size_t)(g * a.Kg + k0 + kl) * a.Cg + c0) * RS + rem] = sum;
    }
}

__global__ __launch_bounds__(256) void reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                            int nsplit, size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = part[i];
    for (int s = 1; s < nsplit; ++s) sum += part[(size_t)s * count + i];
    dw[i] = sum;
}

struct Plan {
    int nsplit;
    size_t ws_bytes;
};

template <int TH, int TW, int KB, int CB, int IMG>
Plan make_plan(const Problem& pr, WgradArgs& a) {
    a.tiles_h = (pr.P + TH - 1) / TH;
    a.tiles_w = (pr.Q + TW - 1) / TW;
    a.kblocks = (pr.Kg + 16 * KB - 1) / (16 * KB);
    a.cblocks = (pr.Cg + 16 * CB - 1) / (16 * CB);
    a.img_stages = (pr.N + IMG - 1) / IMG;
    a.stages = a.tiles_h * a.tiles_w * a.img_stages;
    const int blocks = a.kblocks * a.cblocks * pr.groups;
    // Enough workgroups to cover the 256 CUs, but never more partial buffers than stages.
    int nsplit = (256 + blocks - 1) / blocks;
    if (nsplit > a.stages) nsplit = a.stages;
    if (nsplit < 1) nsplit = 1;
    a.nsplit = nsplit;
    a.total_wgs = blocks * nsplit;
    // XCD rectangles: only when the block grid splits exactly into 8 equal rectangles.
    a.xk = a.xc = 0;
    if (nsplit == 1 && pr.groups == 1 && blocks % 8 == 0) {
        const int per = blocks / 8;
        int best = 0;
        for (int xk = 1; xk * xk <= per; ++xk) {
            if (per % xk) continue;
            const int xc = per / xk;
            if (a.kblocks % xk == 0 && a.cblocks % xc == 0 && (a.kblocks / xk) * (a.cblocks / xc) == 8) best = xk;
        }
        if (best) { a.xk = best; a.xc = per / best; }
    }
    const size_t wbytes = (size_t)pr.K * pr.Cg * pr.R * pr.S * sizeof(float);
    return Plan{nsplit, nsplit > 1 ? nsplit * wbytes : 0};
}

// WS: pixel-step shares (waves) on the 16-byte fetch path; WSN: on the 4-byte path, which needs more
// registers per thread and therefore runs one wave per SIMD.
template <typename T, int R, int S, int ST, int TH, int TW, int KB, int CB, int WK, int WC, int WS, int WSN, int IMG>
hipError_t launch_wgrad(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st,
                        bool dry, size_t* ws_bytes) {
    WgradArgs a{};
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.K = pr.K; a.P = pr.P; a.Q = pr.Q;
    a.Cg = pr.Cg; a.Kg = pr.Kg; a.groups = pr.groups; a.pad_h = pr.ph; a.pad_w = pr.pw;
    const Plan pl = make_plan<TH, TW, KB, CB, IMG>(pr, a);
    *ws_bytes = pl.ws_bytes;
    if (dry) return hipSuccess;
    a.out = pl.nsplit > 1 ? static_cast<float*>(ws) : dw;
    const int grid = ((a.total_wgs + 7) / 8) * 8;
    const bool wide = sizeof(T) == 4 && pr.P == TH && pr.Q == TW && (pr.H * pr.W) % 4 == 0 &&
                      pr.H * pr.W == TH * TW * ST * ST;
    if (wide) wgrad_kernel<T, R, S, ST, TH, TW, KB, CB, WK, WC, WS, IMG, true><<<grid, 64 * WK * WC * WS, 0, st>>>(a);
    else wgrad_kernel<T, R, S, ST, TH, TW, KB, CB, WK, WC, WSN, IMG, false><<<grid, 64 * WK * WC * WSN, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1) return e;
    const size_t count = (size_t)pr.K * pr.Cg * pr.R * pr.S;
    reduce_splits_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(static_cast<const float*>(ws), dw,
                                                                          pl.nsplit, count);
    return hipGetLastError();
}

template <typename T>
bool dispatch_wgrad(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st, bool dry,
                    size_t* ws_bytes, hipError_t* err) {
    *err = hipSuccess;
    *ws_bytes = 0;
    if (pr.sh != pr.sw) return false;
    if (pr.R == 3 && pr.S == 3 && pr.sh == 1) {
        *err = launch_wgrad<T, 3, 3, 1, 14, 14, 1, 1, 1, 1, 8, 4, 2>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 3 && pr.S == 3 && pr.sh == 2) {
        *err = launch_wgrad<T, 3, 3, 2, 14, 14, 1, 1, 1, 1, 4, 4, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1) {
        *err = launch_wgrad<T, 1, 1, 1, 2, 14, 8, 8, 2, 2, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    return false;
}

}  // namespace

bool wgrad_supports(const Problem& pr, size_t* ws_bytes) {
    hipError_t e;
    return dispatch_wgrad<float>(pr, nullptr, nullptr, nullptr, nullptr, nullptr, true, ws_bytes, &e);
}

hipError_t wgrad_run(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st) {
    hipError_t e = hipErrorNotSupported;
    size_t bytes;
    const bool ok = pr.dtype == 0 ? dispatch_wgrad<float>(pr, x, dy, dw, ws, st, false, &bytes, &e)
                                  : dispatch_wgrad<uint16_t>(pr, x, dy, dw, ws, st, false, &bytes, &e);
    return ok ? e : hipErrorNotSupported;
}

}  // namespace miconv
