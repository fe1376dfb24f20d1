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
#include <type_traits>

namespace miconv {
namespace {


struct WgradArgs {
    const void* x;
    const void* dy;
    float* out;        // dw, or the partial buffer [nsplit][K*Cg*R*S]
    int N, C, H, W, K, P, Q;
    int Cg, Kg, groups;
    int pad_h, pad_w;
    int tiles_h, tiles_w;
    int kblocks, cblocks;  // per group
    int nsplit, stages;    // stages = tiles_h*tiles_w*img_stages, ordered tile-major (image-major when tile_fastest)
    int tile_fastest;      // wide 1x1 path: consecutive stages are the tiles of one image group
    int img_stages;        // ceil(N / images per stage)
    int total_wgs;
    int xk, xc;            // blocks of one XCD form an xk x xc rectangle of the (k, c) block grid (0: linear runs)
};

constexpr int next_2_mod_4(int v) { return v + ((6 - v % 4) % 4); }   // smallest >= v that is 2 mod 4
constexpr int next_odd(int v) { return v | 1; }
constexpr int cmax(int a, int b) { return a > b ? a : b; }

// IMG: images per stage.  With the waves sharing the pixel steps of a stage, two 14x14 images (98 steps)
// divide more evenly than one (49 steps).
// WIDE: the tile is the whole output plane and the planes are multiples of 4 floats: dy rows and x
// planes are then read as 16-byte pieces (a quarter of the address-unit work of 4-byte reads) and the
// x values scattered into the zero-bordered patch, whose border words are written once.
//
// Nothing but MFMAs, LDS accesses, loads and waits may sit in the multiply loop: an ordinary vector
// instruction does not overlap with a running MFMA of its own SIMD, so every address the loop uses is
// a register prepared outside plus an immediate.  That is why the two LDS buffers are handled by two
// instances of the loop (buffer offsets become immediates) and why all LDS store addresses are kept
// in registers.
// OCC: waves per SIMD the register allocation must allow.
template <typename T, int R, int S, int ST, int TH, int TW, int KB, int CB, int WK, int WC, int WS, int IMG, bool WIDE, int OCC>
__global__ __launch_bounds__(64 * WK * WC * WS, OCC) void wgrad_kernel(WgradArgs a) {
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
    constexpr int YROWS = 16 * KB, XROWS = 16 * CB;                     // channels per image
    constexpr int YIMG = YROWS * DS, XIMG = XROWS * XS;                 // floats per image in LDS
    constexpr int STAGE = IMG * (YIMG + XIMG);                          // floats of one stage
    // Lanes with nothing to store write to a word of their own behind the stage (no branch around
    // a store that sits between MFMAs); BSTR is the distance between the two stage buffers.
    constexpr int TRASH = STAGE, BSTR = STAGE + 64;
    static_assert(STAGE % 4 == 0, "16-byte alignment of the second buffer");
    constexpr int OUTSZ = 16 * KB * 16 * CB * RS;                       // accumulator elements of the workgroup
    constexpr int LDSF = cmax(2 * BSTR, WS * OUTSZ);
    static_assert(LDSF * 4 <= 160 * 1024, "LDS budget");
    // Load pieces per thread.  WIDE: consecutive 16-byte pieces of the stage's dy rows and x planes.
    // Otherwise single elements: thread (row, lane-in-row) walks along its row, so that the LDS address
    // of piece m is the thread's base plus a constant.
    constexpr int YLANES = NPX < 64 ? 32 : 64, XLANES = PW <= 16 ? 16 : (PW <= 32 ? 32 : 64);
    static_assert(NT % YLANES == 0 && NT % XLANES == 0, "row walkers");
    constexpr int YRPP = NT / YLANES, XRPP = NT / XLANES;               // rows covered per pass
    constexpr int YCOLP = (NPX + YLANES - 1) / YLANES, YROWP = (IMG * YROWS + YRPP - 1) / YRPP;
    constexpr int XROWP = (IMG * XROWS * PH + XRPP - 1) / XRPP;         // x rows are (image, channel, patch row)
    constexpr int YPT = WIDE ? (IMG * YROWS * NPX / 4 + NT - 1) / NT : YCOLP * YROWP;
    constexpr int XPT = WIDE ? (IMG * XROWS * (NPX * ST * ST) / 4 + NT - 1) / NT : XROWP;
    static_assert(WIDE || PW <= 64, "one lane per patch column");

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
    // FLAT (1x1 filters on the 16-byte path): a tile is TH full rows, a contiguous run inside each plane whose
    // offset goes into the descriptor base; stages may then be ordered image-major (a.tile_fastest).
    constexpr bool FLAT = WIDE && R == 1 && S == 1 && ST == 1;
    // (integer division goes through the vector ALU: readfirstlane tells the compiler the results are
    // wave-uniform, which the descriptor arithmetic of the FLAT path needs)
    const int s_begin0 = (int)((long long)a.stages * sp / a.nsplit), s_end0 = (int)((long long)a.stages * (sp + 1) / a.nsplit);
    const int s_begin = FLAT ? __builtin_amdgcn_readfirstlane(s_begin0) : s_begin0;
    const int s_end = FLAT ? __builtin_amdgcn_readfirstlane(s_end0) : s_end0;

    const T* xg = static_cast<const T*>(a.x);
    const T* dyg = static_cast<const T*>(a.dy);
    const int xplane = a.H * a.W, yplane = a.P * a.Q;
    const T* const tnull = nullptr;

    // ---- gather plans ----------------------------------------------------------------------------
    // Global byte offsets (relative to the first image of a stage; kOob = reads as zero; images past
    // the end of the batch fall outside the descriptor and read as zero) depend on the tile position;
    // the LDS store addresses (in buffer 0) never change.
    unsigned ygo[YPT], xgo[XPT];
    float* ysto[YPT];
    float* xsto[XPT][WIDE ? 4 : 1];
    if constexpr (WIDE) {
#pragma unroll
        for (int m = 0; m < YPT; ++m) {
            const int f = tid + NT * m;
            const int row = (4 * f) / NPX, px = 4 * f - row * NPX;       // row = image-major, then channel
            const int im = row / YROWS, kl = row - im * YROWS;
            // rows are 8-byte aligned in LDS (DS is even, px a multiple of 4)
            ysto[m] = lds + (row < IMG * YROWS ? im * YIMG + kl * DS + px : TRASH + (lane & ~3));
        }
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int f = tid + NT * m;
            constexpr int xq = NPX * ST * ST / 4;   // 16-byte pieces of one channel's share of a stage
            const int pc = f / xq, rem = 4 * (f - pc * xq);
            const int im = pc / XROWS, cl = pc - im * XROWS;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int ih = (rem + e) / a.W, iw = (rem + e) - ih * a.W;
                const int ph = ih + a.pad_h, pw = iw + a.pad_w;
                const bool in = pc < IMG * XROWS && ph >= 0 && ph < PH && pw >= 0 && pw < PW;
                xsto[m][e] = lds + (in ? IMG * YIMG + im * XIMG + cl * XS + ph * PW + pw : TRASH + lane);
            }
        }
    } else {
        const int yr = tid / YLANES, yc = tid - yr * YLANES;
#pragma unroll
        for (int m = 0; m < YPT; ++m) {
            const int row = yr + YRPP * (m / YCOLP), px = yc + YLANES * (m % YCOLP);
            const int im = row / YROWS, kl = row - im * YROWS;
            ysto[m] = lds + (row < IMG * YROWS && px < NPX ? im * YIMG + kl * DS + px : TRASH + lane);
        }
        const int xr = tid / XLANES, xc = tid - xr * XLANES;
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int row = xr + XRPP * m;                               // (image, channel, patch row)
            const int pc = row / PH, ph = row - pc * PH;
            const int im = pc / XROWS, cl = pc - im * XROWS;
            xsto[m][0] = lds + (pc < IMG * XROWS && xc < PW ? IMG * YIMG + im * XIMG + cl * XS + ph * PW + xc : TRASH + lane);
        }
    }
    auto plan = [&](int tile) __attribute__((always_inline)) {
        if constexpr (WIDE) {
            // a channel's share of a stage is contiguous: the whole plane, or TH full rows of a 1x1 layer
            // (then the tile's offset inside the plane is part of the descriptor base)
            constexpr int xq = NPX * ST * ST / 4;
#pragma unroll
            for (int m = 0; m < YPT; ++m) {
                const int f = tid + NT * m;
                const int row = (4 * f) / NPX, px = 4 * f - row * NPX;
                const int im = row / YROWS, kl = row - im * YROWS;
                const bool ok = row < IMG * YROWS && k0 + kl < a.Kg;
                ygo[m] = ok ? (unsigned)((im * a.K + g * a.Kg + k0 + kl) * yplane + px) * 4u : kOob;
            }
#pragma unroll
            for (int m = 0; m < XPT; ++m) {
                const int f = tid + NT * m;
                const int pc = f / xq, rem = 4 * (f - pc * xq);      // plane (image-major, then channel), element
                const int im = pc / XROWS, cl = pc - im * XROWS;
                const bool ok = pc < IMG * XROWS && c0 + cl < a.Cg;
                xgo[m] = ok ? (unsigned)((im * a.C + g * a.Cg + c0 + cl) * xplane + rem) * 4u : kOob;
            }
            return;
        }
        const int ti = tile / a.tiles_w, tj = tile - ti * a.tiles_w;
        const int p0 = ti * TH, q0 = tj * TW;
        const int h0 = p0 * ST - a.pad_h, v0 = q0 * ST - a.pad_w;
        const int yr = tid / YLANES, yc = tid - yr * YLANES;
#pragma unroll
        for (int m = 0; m < YPT; ++m) {
            const int row = yr + YRPP * (m / YCOLP), px = yc + YLANES * (m % YCOLP);
            const int im = row / YROWS, kl = row - im * YROWS;
            const int th = px / TW, tw = px - th * TW;
            const int p = p0 + th, q = q0 + tw;
            const bool ok = row < IMG * YROWS && px < NPX && k0 + kl < a.Kg && p < a.P && q < a.Q;
            ygo[m] = ok ? (unsigned)((im * a.K + g * a.Kg + k0 + kl) * yplane + p * a.Q + q) * (unsigned)sizeof(T) : kOob;
        }
        const int xr = tid / XLANES, xc = tid - xr * XLANES;
#pragma unroll
        for (int m = 0; m < XPT; ++m) {
            const int row = xr + XRPP * m;
            const int pc = row / PH, ph = row - pc * PH;
            const int im = pc / XROWS, cl = pc - im * XROWS;
            const int h = h0 + ph, v = v0 + xc;
            const bool ok = pc < IMG * XROWS && xc < PW && c0 + cl < a.Cg && h >= 0 && h < a.H && v >= 0 && v < a.W;
            xgo[m] = ok ? (unsigned)((im * a.C + g * a.Cg + c0 + cl) * xplane + h * a.W + v) * (unsigned)sizeof(T) : kOob;
        }
    };

    // The fetch of a stage is cut into single load instructions ("pieces") that the MFMA loop issues
    // a few at a time; issued in one burst they back up in the address unit and stall every wave.
    float yreg[WIDE ? 1 : YPT], xreg[WIDE ? 1 : XPT];
    v4u yreg4[WIDE ? YPT : 1], xreg4[WIDE ? XPT : 1];
    constexpr int NPIECES = YPT + XPT;
    rsrc_t yrs, xrs;
    // The stage being fetched runs ahead of the one being multiplied: (f_tile, f_img) is its position.
    const int ntiles = a.tiles_h * a.tiles_w;
    int f_stage = s_begin;
    int f_tile = FLAT ? __builtin_amdgcn_readfirstlane(a.tile_fastest ? s_begin % ntiles : s_begin / a.img_stages) : s_begin / a.img_stages;
    int f_img = FLAT ? __builtin_amdgcn_readfirstlane(a.tile_fastest ? s_begin / ntiles : s_begin - f_tile * a.img_stages)
                     : s_begin - f_tile * a.img_stages;
    auto descriptors = [&]() __attribute__((always_inline)) {
        const int n = f_img * IMG;                           // first image of the stage
        const int left = f_stage < s_end ? a.N - n : 0;      // past the split's end: empty, every load reads zero
        const int have = left < IMG ? left : IMG;
        if constexpr (FLAT) {
            const int toff = __builtin_amdgcn_readfirstlane(f_tile * NPX);
            const int ybytes = (have * a.K * yplane - toff) * (int)sizeof(T), xbytes = (have * a.C * xplane - toff) * (int)sizeof(T);
            yrs = make_rsrc(dyg + (size_t)n * a.K * yplane + toff, (unsigned)__builtin_amdgcn_readfirstlane(ybytes > 0 ? ybytes : 0));
            xrs = make_rsrc(xg + (size_t)n * a.C * xplane + toff, (unsigned)__builtin_amdgcn_readfirstlane(xbytes > 0 ? xbytes : 0));
        } else {
            yrs = make_rsrc(dyg + (size_t)n * a.K * yplane, (unsigned)(have * a.K * yplane) * (unsigned)sizeof(T));
            xrs = make_rsrc(xg + (size_t)n * a.C * xplane, (unsigned)(have * a.C * xplane) * (unsigned)sizeof(T));
        }
    };
    auto advance = [&]() __attribute__((always_inline)) {   // to the next stage to fetch (wave-uniform arithmetic only)
        ++f_stage;
        if constexpr (FLAT) {
            // (written with selects on values: a select between the two counters' addresses would put them in memory)
            const bool tf = a.tile_fastest != 0;
            const int inner = (tf ? f_tile : f_img) + 1;
            const bool wrap = inner == (tf ? ntiles : a.img_stages);
            const int inner2 = wrap ? 0 : inner;
            const int outer2 = (tf ? f_img : f_tile) + (wrap ? 1 : 0);
            f_tile = tf ? inner2 : outer2;
            f_img = tf ? outer2 : inner2;
        } else if (++f_img == a.img_stages) {
            f_img = 0;
            ++f_tile;
            if (!WIDE && f_stage < s_end) plan(f_tile);
        }
        descriptors();
    };
    auto issue = [&](int piece) __attribute__((always_inline)) {
        if constexpr (WIDE) {
            if (piece < YPT) yreg4[piece] = __builtin_amdgcn_raw_buffer_load_b128(yrs, ygo[piece], 0, 0);
            else xreg4[piece - YPT] = __builtin_amdgcn_raw_buffer_load_b128(xrs, xgo[piece - YPT], 0, 0);
        } else {
            if (piece < YPT) yreg[piece] = buf_load(yrs, ygo[piece], tnull);
            else xreg[piece - YPT] = buf_load(xrs, xgo[piece - YPT], tnull);
        }
    };
    // LDS stores of one fetched piece (its load must have completed) into buffer `buf` (a constant).
    auto write_piece = [&](int piece, int buf) __attribute__((always_inline)) {
        const int bo = buf * BSTR;
        if constexpr (WIDE) {
            if (piece < YPT) {
                const int m = piece;
                *reinterpret_cast<float2*>(ysto[m] + bo) = make_float2(__uint_as_float(yreg4[m].x), __uint_as_float(yreg4[m].y));
                *reinterpret_cast<float2*>(ysto[m] + bo + 2) = make_float2(__uint_as_float(yreg4[m].z), __uint_as_float(yreg4[m].w));
            } else {
                const int m = piece - YPT;
#pragma unroll
                for (int e = 0; e < 4; ++e) xsto[m][e][bo] = __uint_as_float(xreg4[m][e]);
            }
        } else {
            if (piece < YPT) ysto[piece][bo] = yreg[piece];
            else xsto[piece - YPT][0][bo] = xreg[piece - YPT];
        }
    };

    v4f acc[KBW][CBW][RS];
#pragma unroll
    for (int i = 0; i < KBW; ++i)
#pragma unroll
        for (int j = 0; j < CBW; ++j)
#pragma unroll
            for (int t = 0; t < RS; ++t) acc[i][j][t] = v4f{0.f, 0.f, 0.f, 0.f};

    // ---- this wave's pixel steps; the LDS addresses of its lanes never change -------------------
    // Wave ws takes steps ws, ws+WS, ...
    constexpr int ITER = (NSTEPS + WS - 1) / WS;
    constexpr int MINCNT = NSTEPS / WS;   // steps every wave runs
    const int mycnt = __builtin_amdgcn_readfirstlane(NSTEPS / WS + (ws < NSTEPS % WS ? 1 : 0));
    const float* yrd[ITER];
    const float* xrd[ITER];
#pragma unroll
    for (int i = 0; i < ITER; ++i) {
        int t = ws + WS * i;
        if (t >= NSTEPS) t = NSTEPS - 1;   // steps beyond this wave's count are skipped; keeps their reads in range
        const int im = t / SPI;
        const int px = 4 * (t - im * SPI) + kk;
        const int th = px / TW, tw = px - th * TW;
        yrd[i] = lds + im * YIMG + (16 * (wk * KBW) + li) * DS + px;
        xrd[i] = lds + IMG * YIMG + im * XIMG + (16 * (wc * CBW) + li) * XS + th * ST * PW + tw * ST;
    }

    // One step = NM = KBW*CBW*RS MFMAs on NR = KBW + CBW*RS operands.  Operand r of step i+1 is read
    // from LDS in the slot of MFMA r of step i, so reads issue while the matrix pipe is busy and every
    // operand is requested a full step before its use; scheduling fences pin that order.
    constexpr int NM = KBW * CBW * RS, NR = KBW + CBW * RS;
    // Software pipeline over stages, all inside the MFMA loop so that no wave ever leaves it for a
    // separate copy phase: while stage s is multiplied, the registers hold stage s+1 (fetched during
    // stage s-1); the first third of the steps stores them, a few LDS stores behind each MFMA, into
    // the other LDS buffer; the second third refills the registers with the loads of stage s+2; the
    // last third covers the latency of those loads.
    constexpr int SLOTS = NM > NR ? NM : NR;
    constexpr int WSTEPS = ITER >= 3 ? ITER / 3 : 1;
    constexpr int ISSUE_STEPS = ITER >= 3 ? ITER / 3 : 1;
    static_assert(ITER == 1 || WSTEPS + ISSUE_STEPS <= ITER, "store steps, then load steps");
    static_assert(WSTEPS <= MINCNT, "the stores lie in steps every wave runs");
    // buf: the LDS buffer multiplied (a constant at each call site); the other one is stored to.
    auto multiply = [&](auto bufc) __attribute__((always_inline)) {
        constexpr int buf = decltype(bufc)::value;
        constexpr int bo = buf * BSTR;
        float ops[2][NR];   // [0..KBW): dy operands, then CBW*RS x operands
        auto read_op = [&](int i, int r) __attribute__((always_inline)) -> float {
            if (r < KBW) return yrd[i][bo + r * 16 * DS];
            const int q = r - KBW, j = q / RS, t = q % RS;
            return xrd[i][bo + j * 16 * XS + (t / S) * PW + (t % S)];
        };
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the held stage was requested two thirds of a stage ago
#pragma unroll
        for (int r = 0; r < NR; ++r) ops[0][r] = read_op(0, r);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < ITER; ++i) {
            // Steps past MINCNT exist only for some waves (wave-uniform test).  Once the stores and loads
            // of the stage are out, such a wave leaves the loop; before that it only skips the MFMAs.
            if (i >= MINCNT && i >= WSTEPS + ISSUE_STEPS && i >= mycnt) break;
            const bool next = i + 1 < ITER;
            if (i < MINCNT || i >= WSTEPS + ISSUE_STEPS || i < mycnt) {
#pragma unroll
                for (int m = 0; m < SLOTS; ++m) {
                    if (next && m < NR) ops[(i + 1) & 1][m] = read_op(i + 1, m);
                    if (m < NM) {
                        const int j = m / (RS * KBW), t = (m / KBW) % RS, ib = m % KBW;
                        acc[ib][j][t] = __builtin_amdgcn_mfma_f32_16x16x4f32(ops[i & 1][ib], ops[i & 1][KBW + j * RS + t],
                                                                             acc[ib][j][t], 0, 0, 0);
                    }
                    {   // pieces p with floor(p * WACT / NPIECES) == this slot's index
                        constexpr int WACT = WSTEPS * SLOTS;
                        const int act = i * SLOTS + m;
                        const int lo = (act * NPIECES + WACT - 1) / WACT, hi = ((act + 1) * NPIECES + WACT - 1) / WACT;
#pragma unroll
                        for (int d = 0; d < (NPIECES + WACT - 1) / WACT + 1; ++d)
                            if (act < WACT && lo + d < hi && lo + d < NPIECES) write_piece(lo + d, buf ^ 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            // loads go out behind the stores of the same registers
            {   // pieces p with floor(p * ISSUE_STEPS / NPIECES) == k
                const int k = ITER == 1 ? 0 : i - WSTEPS;
                const int lo = (k * NPIECES + ISSUE_STEPS - 1) / ISSUE_STEPS, hi = ((k + 1) * NPIECES + ISSUE_STEPS - 1) / ISSUE_STEPS;
#pragma unroll
                for (int d = 0; d < (NPIECES + ISSUE_STEPS - 1) / ISSUE_STEPS + 1; ++d)
                    if (k >= 0 && k < ISSUE_STEPS && lo + d < hi && lo + d < NPIECES) issue(lo + d);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // patch borders (and everything else) start as zero; the wide scatter only writes interior words
    for (int e = tid; e < LDSF; e += NT) lds[e] = 0.f;
    __syncthreads();
    if (s_begin < s_end) {
        plan(f_tile);
        descriptors();
#pragma unroll
        for (int piece = 0; piece < NPIECES; ++piece) issue(piece);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
#pragma unroll
        for (int piece = 0; piece < NPIECES; ++piece) write_piece(piece, 0);
        advance();   // stage s_begin+1 into the registers
#pragma unroll
        for (int piece = 0; piece < NPIECES; ++piece) issue(piece);
        __syncthreads();
        for (int stage = s_begin; stage < s_end; stage += 2) {
            advance();
            multiply(std::integral_constant<int, 0>{});
            __syncthreads();
            if (stage + 1 >= s_end) break;
            advance();
            multiply(std::integral_constant<int, 1>{});
            __syncthreads();
        }
    }

    // ---- combine the WS pixel-step shares and write out ---------------------------------------------
    // LDS layout of one share: [k local][c local][tap], i.e. the order of dw within the block.
    __builtin_amdgcn_s_waitcnt(0x0F70);   // loads fetched past the last stage still target registers
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
    // in split order, eight loads in flight at a time
    float sum = part[i];
    int s = 1;
    for (; s + 8 <= nsplit; s += 8) {
        float v[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = part[(size_t)(s + k) * count + i];
#pragma unroll
        for (int k = 0; k < 8; ++k) sum += v[k];
    }
    float v[7];
#pragma unroll
    for (int k = 0; k < 7; ++k) v[k] = s + k < nsplit ? part[(size_t)(s + k) * count + i] : 0.f;
#pragma unroll
    for (int k = 0; k < 7; ++k) sum += v[k];
    dw[i] = sum;
}

struct Plan {
    int nsplit;
    size_t ws_bytes;
};

template <int TH, int TW, int KB, int CB, int IMG, int OCC>
Plan make_plan(const Problem& pr, WgradArgs& a) {
    a.tiles_h = (pr.P + TH - 1) / TH;
    a.tiles_w = (pr.Q + TW - 1) / TW;
    a.kblocks = (pr.Kg + 16 * KB - 1) / (16 * KB);
    a.cblocks = (pr.Cg + 16 * CB - 1) / (16 * CB);
    a.img_stages = (pr.N + IMG - 1) / IMG;
    a.stages = a.tiles_h * a.tiles_w * a.img_stages;
    const int blocks = a.kblocks * a.cblocks * pr.groups;
    // Enough workgroups to cover the 256 CUs OCC times, but never more partial buffers than stages.
    int nsplit = (256 * OCC + blocks - 1) / blocks;
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
// WS, IMG: pixel-step shares (waves) and images per stage on the 16-byte fetch path; WSN, IMGN: on the 4-byte path.
template <typename T, int R, int S, int ST, int TH, int TW, int KB, int CB, int WK, int WC, int WS, int WSN, int IMG, int OCC = 1,
          int IMGN = IMG>
hipError_t launch_wgrad(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st,
                        bool dry, size_t* ws_bytes) {
    WgradArgs a{};
    a.x = x; a.dy = dy;
    a.N = pr.N; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.K = pr.K; a.P = pr.P; a.Q = pr.Q;
    a.Cg = pr.Cg; a.Kg = pr.Kg; a.groups = pr.groups; a.pad_h = pr.ph; a.pad_w = pr.pw;
    // 16-byte fetch path: a channel's share of a stage is one contiguous run - the whole plane, or (1x1
    // filters without padding) TH full rows of it
    const bool whole = pr.P == TH && pr.Q == TW && pr.H * pr.W == TH * TW * ST * ST;
    const bool rows = R == 1 && S == 1 && ST == 1 && pr.ph == 0 && pr.pw == 0 && pr.Q == TW && pr.P % TH == 0;
    const bool wide_shape = sizeof(T) == 4 && (pr.H * pr.W) % 4 == 0 && (pr.P * pr.Q) % 4 == 0 && (TH * TW) % 4 == 0 && (whole || rows);
    if (dry) {   // the pointers (their alignment picks the path) are not known yet: report the larger need
        WgradArgs b = a;
        const Plan p1 = make_plan<TH, TW, KB, CB, IMG, OCC>(pr, a), p2 = make_plan<TH, TW, KB, CB, IMGN, 1>(pr, b);
        *ws_bytes = p1.ws_bytes > p2.ws_bytes ? p1.ws_bytes : p2.ws_bytes;
        return hipSuccess;
    }
    const bool aligned = reinterpret_cast<uintptr_t>(x) % 16 == 0 && reinterpret_cast<uintptr_t>(dy) % 16 == 0;
    const bool wide = wide_shape && aligned;
    const Plan pl = wide ? make_plan<TH, TW, KB, CB, IMG, OCC>(pr, a) : make_plan<TH, TW, KB, CB, IMGN, 1>(pr, a);
    *ws_bytes = pl.ws_bytes;
    a.out = pl.nsplit > 1 ? static_cast<float*>(ws) : dw;
    const int grid = ((a.total_wgs + 7) / 8) * 8;
    a.tile_fastest = wide && !whole;
    if (wide) wgrad_kernel<T, R, S, ST, TH, TW, KB, CB, WK, WC, WS, IMG, true, (WK * WC * WS + 3) / 4 * OCC><<<grid, 64 * WK * WC * WS, 0, st>>>(a);
    else wgrad_kernel<T, R, S, ST, TH, TW, KB, CB, WK, WC, WSN, IMGN, false, (WK * WC * WSN + 3) / 4><<<grid, 64 * WK * WC * WSN, 0, st>>>(a);
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
    // The kernel forms 32-bit byte offsets relative to the first image of a stage (at most four images) and
    // uses offsets from 2^31 on as "reads zero": a stage's channels must stay below that.
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if (4 * (size_t)pr.C * pr.H * pr.W * esz >= lim || 4 * (size_t)pr.K * pr.P * pr.Q * esz >= lim) return false;
    if (pr.R == 3 && pr.S == 3 && pr.sh == 1 && pr.P <= 7 && pr.Q <= 7) {
        // planes of at most 7 x 7 pixels: stages of four images x 7 x 8 pixels (the eighth column lies outside the image)
        *err = launch_wgrad<T, 3, 3, 1, 7, 8, 1, 1, 1, 1, 8, 8, 4>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 3 && pr.S == 3 && pr.sh == 1) {
        // Blocks of 32 x 32 channels (four waves own a 16 x 16 block each, two shares of the pixel steps, one image per
        // stage) where the work is enough for 32 stages per workgroup: every dy and x value is then fetched and stored
        // to LDS for twice the MFMAs (512 channels at 28 x 28, N=64: 1792 -> 1604 us; 64 channels at 224 x 224: 2060 ->
        // 1884 us).  Smaller layers keep 16 x 16 blocks: on 256 channels at 14 x 14, N=64, both run 115 us, and only the
        // larger blocks need a split reduction there.
        const long long stages = (long long)pr.N * ((pr.P + 13) / 14) * ((pr.Q + 13) / 14);
        const long long blocks32 = (long long)(pr.Kg / 32) * (pr.Cg / 32) * pr.groups;
        if (pr.Kg % 32 == 0 && pr.Cg % 32 == 0 && stages * blocks32 >= 8192) {
            *err = launch_wgrad<T, 3, 3, 1, 14, 14, 2, 2, 2, 2, 2, 2, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
            return true;
        }
        *err = launch_wgrad<T, 3, 3, 1, 14, 14, 1, 1, 1, 1, 8, 8, 2>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 3 && pr.S == 3 && pr.sh == 2) {
        *err = launch_wgrad<T, 3, 3, 2, 14, 14, 1, 1, 1, 1, 8, 8, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 2) {
        // 128 x 128 channel blocks where both channel counts fill them (256 -> 512 channels, 56 -> 28, N=64: 233 -> 164 us)
        if (pr.Kg > 64 && pr.Cg > 64) *err = launch_wgrad<T, 1, 1, 2, 2, 14, 8, 8, 2, 2, 2, 2, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        else *err = launch_wgrad<T, 1, 1, 2, 2, 14, 4, 4, 2, 2, 2, 2, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1 && pr.P <= 7 && pr.Q <= 7) {
        // 128 output x 64 input channels per workgroup (512 <-> 2048 channels, N=64: 111 -> 91 us; 128 x 128 blocks: 146 us)
        if (pr.Kg > 64) *err = launch_wgrad<T, 1, 1, 1, 7, 8, 8, 4, 2, 2, 2, 2, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        else *err = launch_wgrad<T, 1, 1, 1, 7, 8, 4, 4, 2, 2, 2, 2, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1 && (pr.Cg <= 64 || pr.Kg <= 64) && pr.ph == 0 && pr.pw == 0 &&
        (pr.Q == 28 || pr.Q == 56)) {
        // few channels on wide planes: stages of 112 pixels in full rows, fetched 16 bytes per lane
        if (pr.Q == 28) *err = launch_wgrad<T, 1, 1, 1, 4, 28, 4, 4, 2, 2, 2, 1, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        else *err = launch_wgrad<T, 1, 1, 1, 2, 56, 4, 4, 2, 2, 2, 1, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1 && pr.ph == 0 && pr.pw == 0 && (pr.Q == 28 || pr.Q == 56) && pr.Cg > 64 && pr.Kg > 64) {
        // many channels on wide planes: stages of 56 pixels in full rows
        if (pr.Q == 28) *err = launch_wgrad<T, 1, 1, 1, 2, 28, 8, 4, 2, 2, 2, 1, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        else *err = launch_wgrad<T, 1, 1, 1, 1, 56, 8, 4, 2, 2, 2, 1, 1, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1 && (pr.Cg <= 64 || pr.Kg <= 64)) {
        // few channels: 64 x 64 channel blocks (a 128 x 128 block would be mostly empty)
        *err = launch_wgrad<T, 1, 1, 1, 2, 14, 4, 4, 2, 2, 2, 1, 2, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
        return true;
    }
    if (pr.R == 1 && pr.S == 1 && pr.sh == 1) {
        // 128 output x 64 input channels per workgroup: twice the workgroups of 128 x 128 blocks, so half the partial
        // results to add afterwards (1024 -> 256 channels, 14 x 14, N=64: 67.5 -> 62.5 us; 512 -> 512, N=128: 114 -> 112 us)
        *err = launch_wgrad<T, 1, 1, 1, 2, 14, 8, 4, 2, 2, 2, 1, 2, 1, 1>(pr, x, dy, dw, ws, st, dry, ws_bytes);
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
