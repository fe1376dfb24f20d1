// Convolutions with very few input channels and a large, strided filter (the first layer of an
// AlexNet-style network: C = 3, 11x11, stride 4; forward and backward-weight also for the 7x7 stride-2
// first layer of a ResNet) on the fp32 matrix cores.
//
// With C = 3 there is no channel dimension worth contracting over, so the MFMA K dimension runs
// along the filter row instead: one step multiplies 4 consecutive taps s = 4u .. 4u+3 of one (c, r)
// filter row.  The whole input patch of a tile (all C channels) sits in LDS; lane group kk reads the
// patch at "+kk", so the per-step part of every LDS address is a compile-time immediate.  A filter
// row of S taps takes ceil(S/4) steps, the taps past S carrying zero weights.
//
//   forward          M = 16 filters (A: weights, held in registers for the whole kernel),
//                    N = 16 output pixels (B: patch), K = 4 taps.
//   backward-weight  M = 16 filters (A: dy), N = 16 consecutive taps of the flattened (c, r, s) order
//                    (B: patch at a per-lane tap offset), K = 4 output pixels of one output row.
//                    Stages (image x pixel tile) are shared out over the workgroups; the partial
//                    filters are summed afterwards in a fixed order.
#include "common.h"

#include <type_traits>

namespace miconv {
namespace {


struct SmallArgs {
    const void* x;
    const void* w;     // forward: filters; backward-weight: dy
    float* out;        // forward: y; backward-weight: dw or partial buffer [nsplit][K*C*R*S]
    int N, H, W, K, P, Q;
    int pad_h, pad_w;
    int tiles_h, tiles_w;
    int kblocks;       // blocks of 64 filters
    int nsplit, stages;
    unsigned x_bytes, w_bytes;
};

// ---------------------------------------------------------------------------------------- forward
// Persistent workgroups of eight waves.  A work item is one image x one tile of TH x TW output pixels
// (all filters of the workgroup's 64-filter block); wave (wf, wp) owns 16 filters and half of the
// tile's 16-pixel blocks.  The lane's weights (all C*R filter rows) are loaded once and stay in
// registers.  The patch of item i+1 is requested before item i is multiplied and stored to the other
// LDS buffer afterwards: one barrier per item.  Patch rows are dealt out to the waves, so a row's
// validity and address are scalar (a zero-size descriptor for rows outside the image, the row's
// offset in the scalar offset operand) and no vector ALU work is spent on them.
__device__ __forceinline__ float buf_load_s(rsrc_t r, unsigned byte_off, unsigned soff, const float*) {
    return __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, soff, 0));
}
__device__ __forceinline__ float buf_load_s(rsrc_t r, unsigned byte_off, unsigned soff, const uint16_t*) {
    return __uint_as_float(static_cast<unsigned>(__builtin_amdgcn_raw_buffer_load_b16(r, byte_off, soff, 0)) << 16);
}

template <typename T, int C, int R, int S, int ST, int TH, int TW>
__global__ __launch_bounds__(512) void smallc_fwd_kernel(SmallArgs a) {
    constexpr int NW = 8;
    constexpr int SU = (S + 3) / 4;                 // steps per filter row
    constexpr int NSTEP = C * R * SU;
    constexpr int PH = (TH - 1) * ST + R;
    constexpr int PWR = (TW - 1) * ST + S;          // columns that hold data
    constexpr int PW = (TW - 1) * ST + 4 * SU;      // ... plus the columns the zero-weight taps read
    constexpr int CS = PH * PW;
    constexpr int XE = C * CS;
    constexpr int BUFSZ = XE + 64;                  // + words for lanes that have nothing to store
    constexpr int ROWS = C * PH;                    // patch rows, dealt out to the waves
    constexpr int RPW = (ROWS + NW - 1) / NW;
    constexpr int CPL = (PW + 63) / 64;             // column chunks per lane
    constexpr int NPX = TH * TW;
    constexpr int NB = (NPX + 15) / 16;
    constexpr int NB0 = (NB + 1) / 2;               // blocks of the waves with wp = 0; the others take NB - NB0
    constexpr unsigned ESZ = sizeof(T);

    __shared__ float patch[2 * BUFSZ];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = wave & 3, wp = wave >> 2;
    const int li = lane & 15, kk = lane >> 4;
    const int kb = blockIdx.x % a.kblocks, slot = blockIdx.x / a.kblocks, nslots = gridDim.x / a.kblocks;
    const int items = a.N * a.tiles_h * a.tiles_w;
    const T* const tnull = nullptr;

    // ---- this lane's filter values: w[f][c][r][4u+kk], zero past the end of a filter row -----------
    const int f = kb * 64 + wf * 16 + li;
    const rsrc_t wrs = make_rsrc(a.w, a.w_bytes);
    float wa[NSTEP];
#pragma unroll
    for (int st = 0; st < NSTEP; ++st) {
        const int cr = st / SU, uu = st - cr * SU;
        const int s = 4 * uu + kk;
        const bool ok = f < a.K && s < S;
        wa[st] = buf_load(wrs, ok ? (unsigned)((f * C * R + cr) * S + s) * ESZ : kOob, tnull);
    }

    const rsrc_t xrs = make_rsrc(a.x, a.x_bytes), nors = make_rsrc(a.x, 0);
    // where this lane's column chunks go inside a patch row (words); lanes past the row end use a spare word
    int sto[CPL];
#pragma unroll
    for (int j = 0; j < CPL; ++j) sto[j] = lane + 64 * j < PW ? wave * PW + lane + 64 * j : XE + lane;

    float xv[RPW][CPL];
    struct Where { int n, p0, q0; };
    auto decode = [&](int item) __attribute__((always_inline)) -> Where {
        const int tj = item % a.tiles_w, r2 = item / a.tiles_w;
        const int ti = r2 % a.tiles_h;
        return Where{__builtin_amdgcn_readfirstlane(r2 / a.tiles_h), __builtin_amdgcn_readfirstlane(ti * TH),
                     __builtin_amdgcn_readfirstlane(tj * TW)};
    };
    auto issue = [&](int item) __attribute__((always_inline)) {
        const Where wh = decode(item);
        const int h0 = wh.p0 * ST - a.pad_h, v0 = wh.q0 * ST - a.pad_w;
        unsigned colv[CPL];
#pragma unroll
        for (int j = 0; j < CPL; ++j) {
            const int pw = lane + 64 * j, v = v0 + pw;
            colv[j] = pw < PWR && v >= 0 && v < a.W ? (unsigned)v * ESZ : kOob;
        }
#pragma unroll
        for (int k = 0; k < RPW; ++k) {
            const int rr = wave + NW * k;
            const int c = rr / PH, ph = rr - c * PH;
            const int h = h0 + ph;
            const bool ok = rr < ROWS && h >= 0 && h < a.H;
            const rsrc_t rs = ok ? xrs : nors;
            const unsigned soff = ok ? (unsigned)(((wh.n * C + c) * a.H + h) * a.W) * ESZ : 0u;
#pragma unroll
            for (int j = 0; j < CPL; ++j) xv[k][j] = buf_load_s(rs, colv[j], soff, tnull);
        }
    };
    auto store = [&](int buf) __attribute__((always_inline)) {
        float* dst = patch + buf * BUFSZ;
#pragma unroll
        for (int k = 0; k < RPW; ++k) {
            if (wave + NW * k >= ROWS) break;   // scalar
#pragma unroll
            for (int j = 0; j < CPL; ++j) dst[sto[j] + (sto[j] < XE ? k * NW * PW : 0)] = xv[k][j];
        }
    };

    // pixel blocks of this wave: i0 .. i0 + NBW - 1
    const int i0 = wp * NB0;
    int pixoff[NB0];
#pragma unroll
    for (int ii = 0; ii < NB0; ++ii) {
        int j = 16 * (i0 + ii) + li;
        if (j >= NPX) j = 0;
        const int th = j / TW, tw = j - th * TW;
        pixoff[ii] = th * ST * PW + tw * ST + kk;
    }

    // One item on NBW blocks: operand ii of the next step is read from LDS right before MFMA ii of this step.
    auto compute = [&](const float* pb, const Where& wh, auto nbwc) __attribute__((always_inline)) {
        constexpr int NBW = decltype(nbwc)::value;
        v4f acc[NBW];
#pragma unroll
        for (int ii = 0; ii < NBW; ++ii) acc[ii] = v4f{0.f, 0.f, 0.f, 0.f};
        float bq[2][NBW];
#pragma unroll
        for (int ii = 0; ii < NBW; ++ii) bq[0][ii] = pb[pixoff[ii]];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            const int sn = st + 1;
            const int crn = sn / SU, un = sn - crn * SU;
            const int off = (crn / R) * CS + (crn % R) * PW + 4 * un;
#pragma unroll
            for (int ii = 0; ii < NBW; ++ii) {
                if (sn < NSTEP) bq[sn & 1][ii] = pb[pixoff[ii] + off];
                acc[ii] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[st], bq[st & 1][ii], acc[ii], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // ---- D[f = 4*kk+v][pixel = li] -----------------------------------------------------------------
        const int fq = kb * 64 + wf * 16 + 4 * kk;
        float* y = a.out + (size_t)wh.n * a.K * a.P * a.Q;
#pragma unroll
        for (int ii = 0; ii < NBW; ++ii) {
            const int j = 16 * (i0 + ii) + li;
            if (j >= NPX) continue;
            const int th = j / TW, tw = j - th * TW;
            const int p = wh.p0 + th, q = wh.q0 + tw;
            if (p >= a.P || q >= a.Q) continue;
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (fq + v < a.K) y[((size_t)(fq + v) * a.P + p) * a.Q + q] = acc[ii][v];
        }
    };

    int item = slot, buf = 0;
    if (item < items) {
        issue(item);
        store(0);
    }
    __syncthreads();
    for (; item < items; item += nslots) {
        const int next = item + nslots;
        if (next < items) issue(next);   // travels while this item is multiplied
        const Where wh = decode(item);
        const float* pb = patch + buf * BUFSZ;
        if (wp == 0) compute(pb, wh, std::integral_constant<int, NB0>{});
        else compute(pb, wh, std::integral_constant<int, NB - NB0>{});
        if (next < items) store(buf ^ 1);
        __syncthreads();   // the next patch is complete, and every wave is done with this one
        buf ^= 1;
    }
}

// -------------------------------------------------------------------------------- backward-weight
// Workgroup = 64 filters x all C*R*S taps, for a contiguous run of stages; stage = one image x TH
// output rows x TQ4*4 output columns.  The taps of a filter are numbered t = (c*R + r)*S + s and cut
// into blocks of 16 for the MFMA N dimension (363 taps: 23 blocks, against 33 with one block per
// 11-tap filter row).  Lane (li, kk) of block b reads x at "tap offset of 16 b + li" + 4 kk, a value
// it keeps in a register per block; the step (output row, column quad) adds an immediate.  Eight
// waves: wave (wf, wt) owns 16 filters and half of the tap blocks.  Rows of x and dy are dealt out to
// the waves, so their validity and addresses are scalar; the next stage is requested before this one
// is multiplied and stored to the other LDS buffer afterwards.
template <typename T, int C, int R, int S, int ST, int TH, int TQ4>
__global__ __launch_bounds__(512) void smallc_wgrad_kernel(SmallArgs a) {
    constexpr int NW = 8;
    constexpr int TW = 4 * TQ4;                     // output columns of a tile
    constexpr int PH = (TH - 1) * ST + R;
    constexpr int PWR = (TW - 1) * ST + S;          // columns that hold data
    constexpr int PW = (PWR + 3) & ~3;
    constexpr int CS = PH * PW;
    constexpr int XE = C * CS;
    constexpr int YS = TH * TW + 2;                 // dy row stride in LDS: 2 mod 4 keeps the A reads conflict-free
    constexpr int STAGE = XE + 64 * YS + 64;        // + words for lanes that have nothing to store
    constexpr int TRASH = XE + 64 * YS;
    constexpr int NTAP = C * R * S;
    constexpr int NBLK = (NTAP + 15) / 16;          // tap blocks
    constexpr int NB0 = (NBLK + 1) / 2;             // blocks of the waves with wt = 0; the others take NBLK - NB0
    constexpr int OUTSZ = 64 * NBLK * 16;
    constexpr int LDSF = 2 * STAGE > OUTSZ ? 2 * STAGE : OUTSZ;
    constexpr int XROWS = C * PH, XRPW = (XROWS + NW - 1) / NW, XCPL = (PW + 63) / 64;
    constexpr int YROWS = 64 * TH, YRPW = YROWS / NW;
    constexpr unsigned ESZ = sizeof(T);
    static_assert(LDSF * 4 <= 160 * 1024, "LDS budget");
    static_assert((TH * TW) % 4 == 0 && TW <= 64 && YROWS % NW == 0 && YRPW % TH == 0, "tile shape");

    __shared__ float lds[LDSF];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wf = wave & 3, wt = wave >> 2;
    const int li = lane & 15, kk = lane >> 4;
    const int kb = blockIdx.x % a.kblocks, sp = blockIdx.x / a.kblocks;
    const int s_begin = (int)((long long)a.stages * sp / a.nsplit);
    const int s_end = (int)((long long)a.stages * (sp + 1) / a.nsplit);
    const int tiles = a.tiles_h * a.tiles_w;
    const T* const tnull = nullptr;
    const rsrc_t xrs = make_rsrc(a.x, a.x_bytes), nors = make_rsrc(a.x, 0);
    const rsrc_t yrs = make_rsrc(a.w, a.w_bytes);   // dy

    // where this lane's pieces go inside an x row / a dy row (words)
    int xsto[XCPL];
#pragma unroll
    for (int j = 0; j < XCPL; ++j) xsto[j] = lane + 64 * j < PW ? wave * PW + lane + 64 * j : TRASH + lane;
    // dy row d = wave*YRPW + m: filter d / TH, tile row d % TH
    const int ysto = lane < TW ? XE + wave * (YRPW / TH) * YS + lane : TRASH + lane;

    float xv[XRPW][XCPL], yv[YRPW];
    auto fetch = [&](int stage) __attribute__((always_inline)) {
        const int n = __builtin_amdgcn_readfirstlane(stage / tiles), t = stage - n * tiles;
        const int ti = __builtin_amdgcn_readfirstlane(t / a.tiles_w), tj = t - ti * a.tiles_w;
        const int p0 = ti * TH, q0 = tj * TW;
        const int h0 = p0 * ST - a.pad_h, v0 = q0 * ST - a.pad_w;
        const bool live = stage < s_end;
        unsigned colv[XCPL];
#pragma unroll
        for (int j = 0; j < XCPL; ++j) {
            const int pw = lane + 64 * j, v = v0 + pw;
            colv[j] = pw < PWR && v >= 0 && v < a.W ? (unsigned)v * ESZ : kOob;
        }
#pragma unroll
        for (int k = 0; k < XRPW; ++k) {
            const int rr = wave + NW * k;
            const int c = rr / PH, ph = rr - c * PH;
            const int h = h0 + ph;
            const bool ok = live && rr < XROWS && h >= 0 && h < a.H;
            const rsrc_t rs = ok ? xrs : nors;
            const unsigned soff = ok ? (unsigned)(((n * C + c) * a.H + h) * a.W) * ESZ : 0u;
#pragma unroll
            for (int j = 0; j < XCPL; ++j) xv[k][j] = buf_load_s(rs, colv[j], soff, tnull);
        }
        const unsigned ycol = lane < TW && q0 + lane < a.Q ? (unsigned)(q0 + lane) * ESZ : kOob;
#pragma unroll
        for (int m = 0; m < YRPW; ++m) {
            const int d = wave * YRPW + m;
            const int k = kb * 64 + d / TH, p = p0 + d % TH;
            const bool ok = live && k < a.K && p < a.P;
            const rsrc_t rs = ok ? yrs : nors;
            const unsigned soff = ok ? (unsigned)(((n * a.K + k) * a.P + p) * a.Q) * ESZ : 0u;
            yv[m] = buf_load_s(rs, ycol, soff, tnull);
        }
    };
    auto stash = [&](int buf) __attribute__((always_inline)) {
        float* dst = lds + buf * STAGE;
#pragma unroll
        for (int k = 0; k < XRPW; ++k) {
            if (wave + NW * k >= XROWS) break;   // scalar
#pragma unroll
            for (int j = 0; j < XCPL; ++j) dst[xsto[j] + (xsto[j] < XE ? k * NW * PW : 0)] = xv[k][j];
        }
#pragma unroll
        for (int m = 0; m < YRPW; ++m) dst[ysto + (ysto < TRASH ? (m / TH) * YS + (m % TH) * TW : 0)] = yv[m];
    };

    // tap blocks of this wave: b0 .. ; tap t of a lane: offset of x[c][r][s] inside the patch, plus the lane's pixel
    const int b0 = wt * NB0;
    int tapoff[NB0];
#pragma unroll
    for (int m = 0; m < NB0; ++m) {
        const int t = 16 * (b0 + m) + li;
        const int c = t / (R * S), rem = t - c * (R * S);
        const int r = rem / S, ss = rem - r * S;
        tapoff[m] = kk * ST + (t < NTAP ? c * CS + r * PW + ss : 0);   // taps past the last: any valid word, their sums are dropped
    }
    v4f acc[NB0];
#pragma unroll
    for (int m = 0; m < NB0; ++m) acc[m] = v4f{0.f, 0.f, 0.f, 0.f};

    // step = (output row th, column quad uq): pixel = th*TW + 4*uq + kk
    constexpr int NSTEPS = TH * TQ4;
    const int yoff = XE + (wf * 16 + li) * YS + kk;    // A: dy[k = li][pixel]
    auto multiply = [&](const float* xs, auto nbc) __attribute__((always_inline)) {
        constexpr int NBW = decltype(nbc)::value;
        float av[2], bv[2][NBW];
        auto read_ops = [&](int step, float& ao, float (&bo)[NBW], int m) __attribute__((always_inline)) {
            const int th = step / TQ4, uq = step - th * TQ4;
            if (m == 0) ao = xs[yoff + th * TW + 4 * uq];
            bo[m] = xs[tapoff[m] + th * ST * PW + 4 * uq * ST];
        };
#pragma unroll
        for (int m = 0; m < NBW; ++m) read_ops(0, av[0], bv[0], m);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int step = 0; step < NSTEPS; ++step) {
#pragma unroll
            for (int m = 0; m < NBW; ++m) {
                if (step + 1 < NSTEPS) read_ops(step + 1, av[(step + 1) & 1], bv[(step + 1) & 1], m);
                acc[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[step & 1], bv[step & 1][m], acc[m], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };

    if (s_begin < s_end) {
        fetch(s_begin);
        stash(0);
        __syncthreads();
        int buf = 0;
        for (int stage = s_begin; stage < s_end; ++stage) {
            fetch(stage + 1);   // past the end of this workgroup's run: zero-size descriptors, nothing is read
            if (wt == 0) multiply(lds + buf * STAGE, std::integral_constant<int, NB0>{});
            else multiply(lds + buf * STAGE, std::integral_constant<int, NBLK - NB0>{});
            if (stage + 1 < s_end) stash(buf ^ 1);
            __syncthreads();
            buf ^= 1;
        }
    }

    // ---- write the block: LDS transpose to dw order [k][tap], coalesced stores -----------------------------
    __syncthreads();
#pragma unroll
    for (int m = 0; m < NB0; ++m) {
        if (b0 + m >= NBLK) break;   // scalar
#pragma unroll
        for (int v = 0; v < 4; ++v) lds[(wf * 16 + 4 * kk + v) * (NBLK * 16) + 16 * (b0 + m) + li] = acc[m][v];
    }
    __syncthreads();
    float* out = a.out + (a.nsplit > 1 ? (size_t)sp * a.K * NTAP : 0);
    for (int o = tid; o < 64 * NTAP; o += 64 * NW) {
        const int kl = o / NTAP, t = o - kl * NTAP;
        const int k = kb * 64 + kl;
        if (k < a.K) out[(size_t)k * NTAP + t] = lds[kl * (NBLK * 16) + t];
    }
}

// Sum of the partial results in a fixed order: a workgroup of four waves owns 64 elements, wave w adds its quarter of
// the splits in split order (eight loads in flight at a time), and the four sums are added in wave order through LDS.
__global__ __launch_bounds__(256) void smallc_reduce_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                            int nsplit, int count) {
    __shared__ float sh[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane;
    const int s_begin = nsplit * w / 4, s_end = nsplit * (w + 1) / 4;
    float sum = 0.f;
    if (i < count) {
        for (int s0 = s_begin; s0 < s_end; s0 += 8) {
            float v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = s0 + k < s_end ? part[(size_t)(s0 + k) * count + i] : 0.f;
#pragma unroll
            for (int k = 0; k < 8; ++k) sum += v[k];
        }
    }
    sh[w][lane] = sum;
    __syncthreads();
    if (w == 0 && i < count) dw[i] = ((sh[0][lane] + sh[1][lane]) + sh[2][lane]) + sh[3][lane];
}


// ---- backward-data on the vector ALU ------------------------------------------------------------
//   dx[n, c, h, v] = sum_{k, r, s : (h+PAD-r) % ST == 0, (v+PAD-s) % ST == 0} dy[n, k, (h+PAD-r)/ST, (v+PAD-s)/ST] * w[k, c, r, s]
// With C = 3 destination channels an MFMA would use 3 of its 16 rows; the vector ALU has the same
// fp32 peak and no such granularity.  A lane owns an ST x ST block of dx pixels (all C channels):
// each filter tap (r, s) feeds exactly one pixel of that block, from the dy value at a block offset
// that depends on the tap only.  Per output channel k the lane therefore loads the ND x ND dy values
// around its block once (bounds-checked buffer loads: zero outside) and issues C*R*S fused
// multiply-adds whose weight is wave-uniform and comes through the scalar unit (a scalar load feeds
// an SGPR operand).  Nothing is shared between lanes, so a wave needs no LDS and no barrier.
struct SmallBwdArgs {
    const float* dy;
    const float* w;
    float* dx;
    int N, K, H, W, P, Q;
    int btiles_h, btiles_w;   // 8 x 8 blocks of ST x ST pixels per wave
    unsigned dy_bytes;
};

template <int C, int R, int S, int ST, int PAD>
__global__ __launch_bounds__(64) void smallc_bwd_data_kernel(SmallBwdArgs a) {
    // Tap r lands on row phase (r - PAD) mod ST of the block and reads dy row (block row) + dp(r).
    constexpr auto phase = [](int r) { return ((r - PAD) % ST + ST) % ST; };
    constexpr auto dpos = [](int r) { return (((r - PAD) % ST + ST) % ST + PAD - r) / ST; };
    constexpr int DMIN = dpos(R > S ? R - 1 : S - 1), DMAX = dpos(0);   // dpos decreases with r
    constexpr int ND = DMAX - DMIN + 1;
    static_assert(R == S, "square filters");

    int u = blockIdx.x;
    const int tj = u % a.btiles_w; u /= a.btiles_w;
    const int ti = u % a.btiles_h;
    const int n = u / a.btiles_h;
    const int lane = threadIdx.x;
    const int bi = ti * 8 + (lane >> 3), bj = tj * 8 + (lane & 7);   // this lane's block of dx

    const rsrc_t yrs = make_rsrc(a.dy, a.dy_bytes);
    unsigned off[ND][ND];
#pragma unroll
    for (int dr = 0; dr < ND; ++dr)
#pragma unroll
        for (int dc = 0; dc < ND; ++dc) {
            const int p = bi + DMIN + dr, q = bj + DMIN + dc;
            off[dr][dc] = p >= 0 && p < a.P && q >= 0 && q < a.Q ? (unsigned)(p * a.Q + q) * 4u : kOob;
        }
    float acc[C][ST][ST];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int i = 0; i < ST; ++i)
#pragma unroll
            for (int j = 0; j < ST; ++j) acc[c][i][j] = 0.f;

    const unsigned plane = (unsigned)(a.P * a.Q) * 4u;
    unsigned kbase = (unsigned)(n * a.K) * plane;   // byte offset of dy[n, k] (wave-uniform)
    float v[ND][ND], vn[ND][ND];
#pragma unroll
    for (int dr = 0; dr < ND; ++dr)
#pragma unroll
        for (int dc = 0; dc < ND; ++dc)
            v[dr][dc] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(yrs, off[dr][dc], kbase, 0));
    for (int k = 0; k < a.K; ++k) {
        kbase += plane;
        if (k + 1 < a.K) {
#pragma unroll
            for (int dr = 0; dr < ND; ++dr)
#pragma unroll
                for (int dc = 0; dc < ND; ++dc)
                    vn[dr][dc] = __uint_as_float(__builtin_amdgcn_raw_buffer_load_b32(yrs, off[dr][dc], kbase, 0));
        }
        const float* __restrict__ wk = a.w + (size_t)k * (C * R * S);
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int r = 0; r < R; ++r)
#pragma unroll
                for (int s2 = 0; s2 < S; ++s2)
                    acc[c][phase(r)][phase(s2)] =
                        fmaf(v[dpos(r) - DMIN][dpos(s2) - DMIN], wk[(c * R + r) * S + s2], acc[c][phase(r)][phase(s2)]);
#pragma unroll
        for (int dr = 0; dr < ND; ++dr)
#pragma unroll
            for (int dc = 0; dc < ND; ++dc) v[dr][dc] = vn[dr][dc];
    }

    const int h0 = bi * ST, v0 = bj * ST;
    const bool vec = ST == 4 && (a.W & 3) == 0 && (reinterpret_cast<uintptr_t>(a.dx) & 15) == 0;
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int i = 0; i < ST; ++i) {
            const int h = h0 + i;
            if (h >= a.H) continue;
            float* row = a.dx + ((size_t)(n * C + c) * a.H + h) * a.W;
            if (vec && v0 + ST <= a.W) {
                *reinterpret_cast<float4*>(row + v0) = make_float4(acc[c][i][0], acc[c][i][1], acc[c][i][2], acc[c][i][3]);
            } else {
#pragma unroll
                for (int j = 0; j < ST; ++j)
                    if (v0 + j < a.W) row[v0 + j] = acc[c][i][j];
            }
        }
}

// ------------------------------------------------------------------- backward-data on the matrix cores
// dx[n, c, h, w] = sum_{k, r, s} dy[n, k, p, q] w[k, c, r, s] with h + 2 = 4 p + r, w + 2 = 4 q + s
// (11x11, stride 4, padding 2).  Write h = 4 P' + a.  Rows a = 0, 1 see the taps r = a + 2 + 4 j at
// p = P' - j, rows a = 2, 3 the taps r = a - 2 + 4 j at p = P' + 1 - j (j = 0, 1, 2; r = 11 does
// not exist); the same holds for columns.  So the 16 pixel phases (a, b) fall into four groups
// (a / 2, b / 2) whose members read the same dy values, and a group is one GEMM:
//   M = 12 "virtual channels" (c, a % 2, b % 2) in a 16-row MFMA block,
//   N = 16 positions (P', Q'),  K = (k, j_r, j_s) = 64 x 9, four filters per MFMA step.
// 63 % of the multiplications are real (12 of 16 rows, and the taps that do not exist).
// Eight waves: wave = group x half of the tile's position blocks; its A operands (144 per lane)
// stay in registers.  Persistent workgroups walk (image, 2 x 56 positions) items; the dy patch of
// the next item (64 filters x 5 rows x 59 columns) is requested before this one is multiplied and
// stored to the other LDS buffer afterwards.  A lane ends up with 2 x 2 neighbouring pixels of one
// channel and stores them as two 8-byte pairs.
struct SmallBwdMArgs {
    const void* dy;
    const void* w;
    float* dx;
    int N, K, H, W, P, Q;
    int tiles_h, tiles_w;   // tiles of 2 x 56 positions (a position = a 4 x 4 block of pixels)
    int pairs;              // W is even and dx 8-byte aligned
    unsigned dy_bytes, w_bytes;
};

template <typename T>
__global__ __launch_bounds__(512) void smallc_bwd_data_mfma_kernel(SmallBwdMArgs a) {
    constexpr int C = 3, R = 11, S = 11, NW = 8;
    constexpr int TR = 2, TC = 56, NPOS = TR * TC, NB = NPOS / 16, NB0 = (NB + 1) / 2;
    constexpr int PR = TR + 3, PC = TC + 3;         // patch rows p = P0 - 2 .. P0 + TR, columns likewise
    constexpr int PWD = 60, KS = PR * PWD + 4;      // 304 = 16 mod 32: lane groups kk, kk + 1 hit different banks
    constexpr int KF = 64;                          // filters (all of them: K <= 64)
    constexpr int XE = KF * KS, BUFSZ = XE + 64;
    constexpr int ROWS = KF * PR, RPW = ROWS / NW;  // patch rows per wave
    constexpr int NSTEP = (KF / 4) * 9;
    constexpr unsigned ESZ = sizeof(T);
    static_assert(NPOS % 16 == 0 && ROWS % NW == 0 && PC <= 64, "tile shape");
    static_assert(2 * BUFSZ * 4 <= 160 * 1024, "LDS budget");

    __shared__ float patch[2 * BUFSZ];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int grp = wave & 3, wp = wave >> 2;
    const int sa = grp >> 1, sb = grp & 1;
    const int li = lane & 15, kk = lane >> 4;
    const int items = a.N * a.tiles_h * a.tiles_w;
    const T* const tnull = nullptr;

    // ---- A operands: w[k = 4 kq + kk][c][r][s] of virtual channel m = li, zero where the tap does not exist
    const rsrc_t wrs = make_rsrc(a.w, a.w_bytes);
    float wa[NSTEP];
    {
        const int c = li >> 2, al = (li >> 1) & 1, bl = li & 1;
        const int r0 = (2 * sa + al + 2) & 3, s0 = (2 * sb + bl + 2) & 3;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
            const int kq = st / 9, jr = (st % 9) / 3, js = st % 3;
            const int k = 4 * kq + kk, r = r0 + 4 * jr, ss = s0 + 4 * js;
            const bool ok = li < 12 && k < a.K && r < R && ss < S;
            wa[st] = buf_load(wrs, ok ? (unsigned)(((k * C + c) * R + r) * S + ss) * ESZ : kOob, tnull);
        }
    }

    const rsrc_t yrs = make_rsrc(a.dy, a.dy_bytes), nors = make_rsrc(a.dy, 0);
    float xv[RPW];
    struct Where { int n, P0, Q0; };
    auto decode = [&](int item) __attribute__((always_inline)) -> Where {
        const int tj = item % a.tiles_w, r2 = item / a.tiles_w;
        const int ti = r2 % a.tiles_h;
        return Where{__builtin_amdgcn_readfirstlane(r2 / a.tiles_h), __builtin_amdgcn_readfirstlane(ti * TR),
                     __builtin_amdgcn_readfirstlane(tj * TC)};
    };
    auto issue = [&](int item) __attribute__((always_inline)) {
        const Where wh = decode(item);
        const int q = wh.Q0 - 2 + lane;
        const unsigned colv = lane < PC && q >= 0 && q < a.Q ? (unsigned)q * ESZ : kOob;
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int rr = wave + NW * j;
            const int k = rr / PR, pr = rr - k * PR;
            const int p = wh.P0 - 2 + pr;
            const bool ok = k < a.K && p >= 0 && p < a.P;
            xv[j] = buf_load_s(ok ? yrs : nors, colv, ok ? (unsigned)(((wh.n * a.K + k) * a.P + p) * a.Q) * ESZ : 0u, tnull);
        }
    };
    auto store = [&](int buf) __attribute__((always_inline)) {
        float* dst = patch + buf * BUFSZ;
#pragma unroll
        for (int j = 0; j < RPW; ++j) {
            const int rr = wave + NW * j;
            const int k = rr / PR, pr = rr - k * PR;   // scalar
            dst[lane < PC ? k * KS + pr * PWD + lane : XE + lane] = xv[j];
        }
    };

    // position blocks of this wave; lane's position (tr, tc) in block ii and where its dy values start
    const int i0 = wp * NB0;
    int pixoff[NB0];
#pragma unroll
    for (int ii = 0; ii < NB0; ++ii) {
        const int j = 16 * (i0 + ii) + li;
        const int tr = j / TC, tc = j - tr * TC;
        pixoff[ii] = j < NPOS ? kk * KS + (tr + sa) * PWD + tc + sb : 0;
    }

    auto compute = [&](const float* pb, const Where& wh, auto nbwc) __attribute__((always_inline)) {
        constexpr int NBW = decltype(nbwc)::value;
        v4f acc[NBW];
#pragma unroll
        for (int ii = 0; ii < NBW; ++ii) acc[ii] = v4f{0.f, 0.f, 0.f, 0.f};
        // step (kq, jr, js): dy[k][P' + sa - jr][Q' + sb - js] = patch[k][tr + sa - jr + 2][tc + sb - js + 2]
        auto off_of = [](int st) { return (st / 9) * 4 * KS + (2 - (st % 9) / 3) * PWD + (2 - st % 3); };
        float bq[2][NBW];
#pragma unroll
        for (int ii = 0; ii < NBW; ++ii) bq[0][ii] = pb[pixoff[ii] + off_of(0)];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
#pragma unroll
            for (int ii = 0; ii < NBW; ++ii) {
                if (st + 1 < NSTEP) bq[(st + 1) & 1][ii] = pb[pixoff[ii] + off_of(st + 1)];
                acc[ii] = __builtin_amdgcn_mfma_f32_16x16x4f32(wa[st], bq[st & 1][ii], acc[ii], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // ---- D[(c = kk, al, bl) = 4 kk + v][position li]: rows h = 4 P' + 2 sa + al, columns w = 4 Q' + 2 sb + {0, 1}
        if (kk < C) {
            float* dxc = a.dx + ((size_t)wh.n * C + kk) * a.H * a.W;
#pragma unroll
            for (int ii = 0; ii < NBW; ++ii) {
                const int j = 16 * (i0 + ii) + li;
                const int tr = j / TC, tc = j - tr * TC;
                const int h = 4 * (wh.P0 + tr) + 2 * sa, w = 4 * (wh.Q0 + tc) + 2 * sb;
#pragma unroll
                for (int al = 0; al < 2; ++al) {
                    if (h + al >= a.H || w >= a.W) continue;
                    float* row = dxc + (size_t)(h + al) * a.W + w;
                    if (a.pairs) {
                        *reinterpret_cast<float2*>(row) = make_float2(acc[ii][2 * al], acc[ii][2 * al + 1]);
                    } else {
                        row[0] = acc[ii][2 * al];
                        if (w + 1 < a.W) row[1] = acc[ii][2 * al + 1];
                    }
                }
            }
        }
    };

    int item = blockIdx.x, buf = 0;
    if (item < items) {
        issue(item);
        store(0);
    }
    __syncthreads();
    for (; item < items; item += gridDim.x) {
        const int next = item + gridDim.x;
        if (next < items) issue(next);   // travels while this item is multiplied
        const Where wh = decode(item);
        const float* pb = patch + buf * BUFSZ;
        if (wp == 0) compute(pb, wh, std::integral_constant<int, NB0>{});
        else compute(pb, wh, std::integral_constant<int, NB - NB0>{});
        if (next < items) store(buf ^ 1);
        __syncthreads();   // the next patch is complete, and every wave is done with this one
        buf ^= 1;
    }
}

bool shape_ok(const Problem& pr) {
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    return pr.groups == 1 && pr.C == 3 && pr.R == 11 && pr.S == 11 && pr.sh == 4 && pr.sw == 4;
}

// The 7x7 stride-2 first layer of a ResNet: the forward and backward-weight kernels are instantiated for it too.
bool stem_ok(const Problem& pr) {
    const size_t esz = pr.dtype == 0 ? 4 : 2, lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * esz >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * esz >= lim) return false;
    return pr.groups == 1 && pr.C == 3 && pr.R == 7 && pr.S == 7 && pr.sh == 2 && pr.sw == 2;
}

constexpr int kFwdTH = 2, kFwdTW = 55;       // forward tile: two full rows of a 55-wide output
constexpr int kStemTW = 56;                  // ... half a row of the 112-wide output of the 7x7 stride-2 layer
constexpr int kWgTH = 2, kWgTQ4 = 14;        // backward-weight stage: two rows x 56 columns

void fill(const Problem& pr, SmallArgs& a) {
    a.N = pr.N; a.H = pr.H; a.W = pr.W; a.K = pr.K; a.P = pr.P; a.Q = pr.Q; a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.kblocks = (pr.K + 63) / 64;
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    a.x_bytes = (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * esz);
}

int wgrad_splits(const Problem& pr, const SmallArgs& a) {
    int nsplit = 256 / a.kblocks;   // one workgroup per CU
    if (nsplit > a.stages) nsplit = a.stages;
    return nsplit < 1 ? 1 : nsplit;
}

// Backward-data: the padding the kernels are written for; the matrix-core kernel holds all filters (K <= 64), the
// vector-ALU kernel takes fp32 tensors with any number of filters.
bool bwd_mfma_ok(const Problem& pr) { return shape_ok(pr) && pr.ph == 2 && pr.pw == 2 && pr.K <= 64; }
bool stem_bwd_ok(const Problem& pr) { return stem_ok(pr) && pr.dtype == 0 && pr.ph == 3 && pr.pw == 3; }
bool bwd_ok(const Problem& pr) {
    return bwd_mfma_ok(pr) || (shape_ok(pr) && pr.dtype == 0 && pr.ph == 2 && pr.pw == 2) || stem_bwd_ok(pr);
}

}  // namespace

bool smallc_supports(int pass, const Problem& pr) { return pass == 1 ? bwd_ok(pr) : (shape_ok(pr) || stem_ok(pr)); }

size_t smallc_workspace_bytes(int pass, const Problem& pr) {
    if (pass != 2 || !(shape_ok(pr) || stem_ok(pr))) return 0;
    SmallArgs a{};
    fill(pr, a);
    a.tiles_h = (pr.P + kWgTH - 1) / kWgTH; a.tiles_w = (pr.Q + 4 * kWgTQ4 - 1) / (4 * kWgTQ4);
    a.stages = pr.N * a.tiles_h * a.tiles_w;
    const int ns = wgrad_splits(pr, a);
    return ns > 1 ? (size_t)ns * pr.K * pr.C * pr.R * pr.S * sizeof(float) : 0;
}

hipError_t smallc_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws,
                      hipStream_t st) {
    if (!smallc_supports(pass, pr)) return hipErrorNotSupported;
    if (pass == 1 && bwd_mfma_ok(pr)) {
        const unsigned esz = pr.dtype == 0 ? 4 : 2;
        SmallBwdMArgs m{};
        m.dy = in0; m.w = in1; m.dx = out;
        m.N = pr.N; m.K = pr.K; m.H = pr.H; m.W = pr.W; m.P = pr.P; m.Q = pr.Q;
        m.tiles_h = ((pr.H + 3) / 4 + 1) / 2; m.tiles_w = ((pr.W + 3) / 4 + 55) / 56;
        m.pairs = pr.W % 2 == 0 && reinterpret_cast<uintptr_t>(out) % 8 == 0;
        m.dy_bytes = (unsigned)((size_t)pr.N * pr.K * pr.P * pr.Q * esz);
        m.w_bytes = (unsigned)((size_t)pr.K * pr.C * pr.R * pr.S * esz);
        const int items = pr.N * m.tiles_h * m.tiles_w;
        const int grid = items < 256 ? items : 256;   // persistent, one workgroup per CU (its two patch buffers fill the LDS)
        if (pr.dtype == 0) smallc_bwd_data_mfma_kernel<float><<<grid, 512, 0, st>>>(m);
        else smallc_bwd_data_mfma_kernel<uint16_t><<<grid, 512, 0, st>>>(m);
        return hipGetLastError();
    }
    if (pass == 1) {
        SmallBwdArgs b{};
        b.dy = static_cast<const float*>(in0); b.w = static_cast<const float*>(in1); b.dx = out;
        b.N = pr.N; b.K = pr.K; b.H = pr.H; b.W = pr.W; b.P = pr.P; b.Q = pr.Q;
        b.dy_bytes = (unsigned)((size_t)pr.N * pr.K * pr.P * pr.Q * 4);
        if (pr.R == 7) {   // 7x7 stride 2, padding 3: a lane owns a 2 x 2 block of dx pixels
            b.btiles_h = ((pr.H + 1) / 2 + 7) / 8; b.btiles_w = ((pr.W + 1) / 2 + 7) / 8;
            smallc_bwd_data_kernel<3, 7, 7, 2, 3><<<pr.N * b.btiles_h * b.btiles_w, 64, 0, st>>>(b);
            return hipGetLastError();
        }
        b.btiles_h = ((pr.H + 3) / 4 + 7) / 8; b.btiles_w = ((pr.W + 3) / 4 + 7) / 8;
        smallc_bwd_data_kernel<3, 11, 11, 4, 2><<<pr.N * b.btiles_h * b.btiles_w, 64, 0, st>>>(b);
        return hipGetLastError();
    }
    const unsigned esz = pr.dtype == 0 ? 4 : 2;
    SmallArgs a{};
    fill(pr, a);
    a.x = in0;
    if (pass == 0) {
        a.w = in1; a.out = out;
        a.w_bytes = (unsigned)((size_t)pr.K * pr.C * pr.R * pr.S * esz);
        const bool stem = pr.R == 7;
        const int ftw = stem ? kStemTW : kFwdTW;
        a.tiles_h = (pr.P + kFwdTH - 1) / kFwdTH; a.tiles_w = (pr.Q + ftw - 1) / ftw;
        // persistent workgroups, one per CU (two patch buffers take half of its LDS), shared out over the filter blocks
        const int items = pr.N * a.tiles_h * a.tiles_w;
        int slots = 256 / a.kblocks;
        if (slots < 1) slots = 1;
        if (slots > items) slots = items;
        const int grid = slots * a.kblocks;
        if (stem) {
            if (pr.dtype == 0) smallc_fwd_kernel<float, 3, 7, 7, 2, kFwdTH, kStemTW><<<grid, 512, 0, st>>>(a);
            else smallc_fwd_kernel<uint16_t, 3, 7, 7, 2, kFwdTH, kStemTW><<<grid, 512, 0, st>>>(a);
        } else {
            if (pr.dtype == 0) smallc_fwd_kernel<float, 3, 11, 11, 4, kFwdTH, kFwdTW><<<grid, 512, 0, st>>>(a);
            else smallc_fwd_kernel<uint16_t, 3, 11, 11, 4, kFwdTH, kFwdTW><<<grid, 512, 0, st>>>(a);
        }
        return hipGetLastError();
    }
    a.w = in1;   // dy
    a.w_bytes = (unsigned)((size_t)pr.N * pr.K * pr.P * pr.Q * esz);
    a.tiles_h = (pr.P + kWgTH - 1) / kWgTH; a.tiles_w = (pr.Q + 4 * kWgTQ4 - 1) / (4 * kWgTQ4);
    a.stages = pr.N * a.tiles_h * a.tiles_w;
    a.nsplit = wgrad_splits(pr, a);
    a.out = a.nsplit > 1 ? static_cast<float*>(ws) : out;
    const int grid = a.kblocks * a.nsplit;
    if (pr.R == 7) {
        if (pr.dtype == 0) smallc_wgrad_kernel<float, 3, 7, 7, 2, kWgTH, kWgTQ4><<<grid, 512, 0, st>>>(a);
        else smallc_wgrad_kernel<uint16_t, 3, 7, 7, 2, kWgTH, kWgTQ4><<<grid, 512, 0, st>>>(a);
    } else {
        if (pr.dtype == 0) smallc_wgrad_kernel<float, 3, 11, 11, 4, kWgTH, kWgTQ4><<<grid, 512, 0, st>>>(a);
        else smallc_wgrad_kernel<uint16_t, 3, 11, 11, 4, kWgTH, kWgTQ4><<<grid, 512, 0, st>>>(a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.nsplit == 1) return e;
    const int count = pr.K * pr.C * pr.R * pr.S;
    smallc_reduce_kernel<<<(count + 63) / 64, 256, 0, st>>>(static_cast<const float*>(ws), out, a.nsplit, count);
    return hipGetLastError();
}

}  // namespace miconv
