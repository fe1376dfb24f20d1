// Backward-weight 3x3 stride-1 convolution of bf16 tensors on the bf16 matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate, fp32 output), gfx950.
//
//   dw[k, c, r, s] = sum_{n, p, q} dy[n, k, p, q] * x[n, c, p - pad_h + r, q - pad_w + s]
//
// The reduction runs over images and pixels, and an MFMA lane supplies 8 consecutive reduction
// elements of its channel as one 16-byte register group.  If those 8 elements were neighbouring
// pixels, a tap shift of one pixel would misalign every x operand by 2 bytes.  They are therefore
// 8 images at the same pixel: a pre-pass rewrites x and dy into the caller's workspace as
// [N/8][channel][row][column][8 images] (missing images are zeros), after which every tap shift
// is a multiple of 16 bytes and both operands are plain 16-byte LDS reads.
// MFMA roles: M = 16 output channels k (A from dy), N = 16 input channels c (B from x),
// K = 32 = 4 neighbouring pixels x 8 images; one accumulator block per (k block, tap).
//
// Main kernel.  A workgroup owns 64 output channels x 32 input channels (all 9 taps) and a share
// of the "units"; a unit is 8 images x a strip of 28 output columns x a segment of rows.  It walks
// the rows of a unit top to bottom; a stage is one output row.  LDS holds a ring of four x rows
// (three in use, one arriving) and two dy rows, so every x row is fetched once per unit although
// three output rows use it.  Wave (wk, wc) owns 32 k x 16 c: per group of 4 pixels it reads 2 dy
// operands and 9 x operands for 18 MFMAs, which keeps the LDS (the limiter of bf16 MFMA kernels)
// just below saturation.  The row loop is unrolled four times so that ring slots are address
// immediates; the MFMA loop holds no vector-ALU instruction.  Stores of the rows fetched during
// the previous stage and loads of the rows two stages ahead are spread between the MFMAs.
// Partial sums of the splits are added in split order by a second kernel: no float atomics.
#include "common.h"

#include <type_traits>

namespace miconv {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;
constexpr unsigned kOob = 0x80000000u;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, unsigned bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// ---- pre-pass: [N][Ch][HW] -> [ceil(N/8)][Ch][HW][8] ------------------------------------------
struct PackNArgs {
    const uint16_t* src;
    uint16_t* dst;
    int N, Ch, HW;   // HW % 8 == 0
    unsigned src_bytes;
    int total;       // ceil(N/8) * Ch * HW / 8 threads
};

__global__ __launch_bounds__(256) void pack_n8_kernel(PackNArgs a) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= a.total) return;
    const int per = a.HW / 8;
    const int pc = t % per, rest = t / per;
    const int ch = rest % a.Ch, nb = rest / a.Ch;
    const rsrc_t rs = make_rsrc(a.src, a.src_bytes);
    v4u r[8];   // r[i]: 8 consecutive pixels of image nb*8+i
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int n = nb * 8 + i;
        const unsigned off = n < a.N ? (unsigned)((n * a.Ch + ch) * a.HW + 8 * pc) * 2u : kOob;
        r[i] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
    }
    v4u* o = reinterpret_cast<v4u*>(a.dst) + ((size_t)(nb * a.Ch + ch) * a.HW + 8 * pc);
#pragma unroll
    for (int j = 0; j < 8; ++j) {   // pixel j: its value in images 0..7
        v4u v;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const unsigned lo = r[2 * m][j / 2], hi = r[2 * m + 1][j / 2];
            v[m] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        o[j] = v;
    }
}

// ---- main kernel --------------------------------------------------------------------------------
struct BwArgs {
    const uint16_t* xP;    // [NB][C][H][W][8]
    const uint16_t* dyP;   // [NB][K][P][Q][8]
    float* out;            // dw, or partial buffer [nsplit][K][C][9]
    int NB, C, H, W, K, P, Q;
    int pad_h, pad_w;
    int strips, segs, segh;    // unit = (nb, strip, segment); segment height is a multiple of 4
    int kblocks, cblocks, nsplit, units;
    unsigned x_bytes, y_bytes;
};

constexpr int kSQ = 7, kSW = 4 * kSQ, kXW = kSW + 2;   // pixel groups, output columns and x columns per stage
constexpr int kKB = 64, kCB = 32;
constexpr int kDyRow = kSW * 16 + 16;                  // bytes per k in a dy row buffer (464: 20 banks mod 32)
constexpr int kDyBuf = kKB * kDyRow;
constexpr int kXRow = kXW * 16 + 16;                   // bytes per c in an x ring slot (496: 28 banks mod 32)
constexpr int kXSlot = kCB * kXRow;
constexpr int kDyBase = 4 * kXSlot;                    // the ring comes first: its slots are reachable by immediates
constexpr int kLds = kDyBase + 2 * kDyBuf;
constexpr int kYPT = kKB * kSW / 256, kXPT = (kCB * kXW + 255) / 256;
static_assert(kKB * kSW % 256 == 0, "whole dy pieces");
static_assert(3 * kXSlot + kXRow < 65536 && kDyBuf + kDyRow * 16 + kSW * 16 < 65536, "immediate offsets");

__global__ __launch_bounds__(256) void bf16_wgrad_kernel(BwArgs a) {
    constexpr int SLOTS = kSQ * 9, RING = 9, PF = 6;
    static_assert(SLOTS % RING == 0 && PF < RING, "ring");
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];

    const int blocks = a.kblocks * a.cblocks;
    const int blk = blockIdx.x % blocks, sp = blockIdx.x / blocks;
    const int kb = blk / a.cblocks, cb = blk - kb * a.cblocks;
    const int k0 = kb * kKB, c0 = cb * kCB;
    const int u0 = (int)((long long)a.units * sp / a.nsplit), u1 = (int)((long long)a.units * (sp + 1) / a.nsplit);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave & 1, wc = wave >> 1;
    const int li = lane & 15, g = lane >> 4;

    // gather plans; offsets are relative to (image group, first channel of the block, row, first column)
    unsigned ygo[kYPT], xgo[kXPT];
    unsigned char* ysto[kYPT];
    unsigned char* xsto[kXPT];
    int xcol[kXPT], ycol[kYPT];
#pragma unroll
    for (int m = 0; m < kYPT; ++m) {
        const int e = tid + 256 * m;
        const int kl = e / kSW, px = e - kl * kSW;
        ygo[m] = k0 + kl < a.K ? (unsigned)(kl * a.P * a.Q + px) * 16u : kOob;
        ycol[m] = px;
        ysto[m] = lds + kDyBase + kl * kDyRow + px * 16;
    }
#pragma unroll
    for (int m = 0; m < kXPT; ++m) {
        const int e = tid + 256 * m;
        const int cl = e / kXW, xc = e - cl * kXW;
        const bool in = e < kCB * kXW;
        xgo[m] = in && c0 + cl < a.C ? (unsigned)(cl * a.H * a.W) * 16u : kOob;   // the column is added per unit
        xcol[m] = xc;
        // lanes past the last piece store into the unused 16 bytes that end a channel's row
        xsto[m] = lds + (in ? cl * kXRow + xc * 16 : (tid & 31) * kXRow + kXW * 16);
    }
    const unsigned char* ya = lds + kDyBase + (wk * 32 + li) * kDyRow + g * 16;
    const unsigned char* xa = lds + (wc * 16 + li) * kXRow + g * 16;

    v4f acc[2][9];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[i][t] = v4f{0.f, 0.f, 0.f, 0.f};

    const rsrc_t yrs = make_rsrc(a.dyP, a.y_bytes), xrs = make_rsrc(a.xP, a.x_bytes), nors = make_rsrc(a.dyP, 0);
    v4u yreg[kYPT], xreg[kXPT];
    v4u ring[RING], A[2][2];

    for (int unit = u0; unit < u1; ++unit) {
        int u = unit;
        const int seg = u % a.segs; u /= a.segs;
        const int strip = u % a.strips;
        const int nb = u / a.strips;
        const int q0 = strip * kSW;
        const int ps = seg * a.segh, pe = ps + a.segh < a.P ? ps + a.segh : a.P;
        // per-lane column validity of this strip
        unsigned yv[kYPT], xv[kXPT];
#pragma unroll
        for (int m = 0; m < kYPT; ++m) yv[m] = q0 + ycol[m] < a.Q ? ygo[m] : kOob;
#pragma unroll
        for (int m = 0; m < kXPT; ++m) {
            const int col = q0 - a.pad_w + xcol[m];
            xv[m] = col >= 0 && col < a.W && xgo[m] != kOob ? xgo[m] + (unsigned)col * 16u : kOob;
        }
        const unsigned ybase = (unsigned)(((nb * a.K + k0) * a.P) * a.Q + q0) * 16u;   // + row * Q * 16
        const unsigned xbase = (unsigned)((nb * a.C + c0) * a.H * a.W) * 16u;          // + row * W * 16

        // Stage p: store the rows fetched during stage p-1 (dy row p+1, x row p+3-pad_h), multiply output
        // row p, fetch dy row p+2 and x row p+4-pad_h.  The four stages before the first row only fill LDS.
        auto stage = [&](auto phc, int p) __attribute__((always_inline)) {
            constexpr int PH4 = decltype(phc)::value;            // p mod 4
            constexpr int YB = (PH4 & 1) * kDyBuf;               // dy buffer multiplied in this stage
            constexpr int YW = ((PH4 + 1) & 1) * kDyBuf;         // ... and stored to
            constexpr int XWS = ((PH4 + 3) & 3) * kXSlot;        // ring slot stored to
            const int yr = p + 2, xr = p + 4 - a.pad_h;          // rows fetched in this stage
            const bool yok = yr >= ps && yr < pe, xok = xr >= 0 && xr < a.H;
            const rsrc_t yd = yok ? yrs : nors, xd = xok ? xrs : nors;
            const unsigned ys = yok ? ybase + (unsigned)(yr * a.Q) * 16u : 0u;
            const unsigned xso = xok ? xbase + (unsigned)(xr * a.W) * 16u : 0u;
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the held rows were requested a stage ago
            if (p >= ps) {
                // first operands of the stage
#pragma unroll
                for (int i = 0; i < 2; ++i) A[0][i] = *reinterpret_cast<const v4u*>(ya + YB + i * 16 * kDyRow);
#pragma unroll
                for (int s = 0; s < PF; ++s) {
                    const int tap = s % 9, r = tap / 3, sx = tap % 3;
                    ring[s % RING] = *reinterpret_cast<const v4u*>(xa + ((PH4 + r) & 3) * kXSlot + (4 * (s / 9) + sx) * 16);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int s = 0; s < SLOTS; ++s) {
                    const int quad = s / 9, tap = s % 9;
                    if (s + PF < SLOTS) {
                        const int s2 = s + PF, q2 = s2 / 9, t2 = s2 % 9;
                        ring[s2 % RING] = *reinterpret_cast<const v4u*>(xa + ((PH4 + t2 / 3) & 3) * kXSlot + (4 * q2 + t2 % 3) * 16);
                    }
                    if (tap == 2 && quad + 1 < kSQ) {
#pragma unroll
                        for (int i = 0; i < 2; ++i)
                            A[(quad + 1) & 1][i] = *reinterpret_cast<const v4u*>(ya + YB + i * 16 * kDyRow + (quad + 1) * 64);
                    }
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        acc[i][tap] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, A[quad & 1][i]),
                                                                              __builtin_bit_cast(v8bf, ring[s % RING]),
                                                                              acc[i][tap], 0, 0, 0);
                    // rows for the next stage: registers -> LDS in the first third of the slots, then the
                    // same registers are refilled with the rows for the stage after it
#pragma unroll
                    for (int m = 0; m < kYPT; ++m) {
                        if (m * 2 == s) *reinterpret_cast<v4u*>(ysto[m] + YW) = yreg[m];
                        if (21 + m * 2 == s) yreg[m] = __builtin_amdgcn_raw_buffer_load_b128(yd, yv[m], ys, 0);
                    }
#pragma unroll
                    for (int m = 0; m < kXPT; ++m) {
                        if (14 + m * 2 == s) *reinterpret_cast<v4u*>(xsto[m] + XWS) = xreg[m];
                        if (35 + m * 2 == s) xreg[m] = __builtin_amdgcn_raw_buffer_load_b128(xd, xv[m], xso, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int m = 0; m < kYPT; ++m) *reinterpret_cast<v4u*>(ysto[m] + YW) = yreg[m];
#pragma unroll
                for (int m = 0; m < kXPT; ++m) *reinterpret_cast<v4u*>(xsto[m] + XWS) = xreg[m];
#pragma unroll
                for (int m = 0; m < kYPT; ++m) yreg[m] = __builtin_amdgcn_raw_buffer_load_b128(yd, yv[m], ys, 0);
#pragma unroll
                for (int m = 0; m < kXPT; ++m) xreg[m] = __builtin_amdgcn_raw_buffer_load_b128(xd, xv[m], xso, 0);
            }
            __syncthreads();
        };

        // before the unit's first stage the registers must hold defined values (they are stored, unused)
#pragma unroll
        for (int m = 0; m < kYPT; ++m) yreg[m] = v4u{0, 0, 0, 0};
#pragma unroll
        for (int m = 0; m < kXPT; ++m) xreg[m] = v4u{0, 0, 0, 0};
        __syncthreads();   // the previous unit's last reads are done before its rows are overwritten
        for (int p = ps - 4; p < pe; p += 4) {   // ps is a multiple of 4
            stage(std::integral_constant<int, 0>{}, p);
            if (p + 1 >= pe) break;
            stage(std::integral_constant<int, 1>{}, p + 1);
            if (p + 2 >= pe) break;
            stage(std::integral_constant<int, 2>{}, p + 2);
            if (p + 3 >= pe) break;
            stage(std::integral_constant<int, 3>{}, p + 3);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);   // rows fetched past the last stage still target registers

    // ---- write out: D[k = 4*g+v][c = li] of block i, tap t ---------------------------------------------
    const size_t wsize = (size_t)a.K * a.C * 9;
    float* out = a.out + (a.nsplit > 1 ? (size_t)sp * wsize : 0);
    const int c = c0 + wc * 16 + li;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int k = k0 + wk * 32 + i * 16 + 4 * g + v;
            if (k < a.K && c < a.C) {
#pragma unroll
                for (int t = 0; t < 9; ++t) out[((size_t)k * a.C + c) * 9 + t] = acc[i][t][v];
            }
        }
}

__global__ __launch_bounds__(256) void bf16_reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                 int nsplit, size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = part[i];
    for (int s = 1; s < nsplit; ++s) sum += part[(size_t)s * count + i];
    dw[i] = sum;
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Plan {
    int NB, strips, segs, segh, kblocks, cblocks, nsplit, units;
    size_t x_bytes, y_bytes, part_bytes;
};

bool make_plan(const Problem& pr, Plan& pl) {
    if (pr.dtype != 1 || pr.R != 3 || pr.S != 3 || pr.sh != 1 || pr.sw != 1 || pr.groups != 1) return false;
    if (pr.ph > 2 || pr.pw > 2) return false;
    if ((pr.H * pr.W) % 8 != 0 || (pr.P * pr.Q) % 8 != 0) return false;
    pl.NB = (pr.N + 7) / 8;
    pl.x_bytes = (size_t)pl.NB * pr.C * pr.H * pr.W * 16;
    pl.y_bytes = (size_t)pl.NB * pr.K * pr.P * pr.Q * 16;
    const size_t lim = (size_t)1 << 31;
    if (pl.x_bytes >= lim || pl.y_bytes >= lim) return false;
    pl.strips = (pr.Q + kSW - 1) / kSW;
    pl.segh = pr.P >= 112 ? 56 : ((pr.P + 3) / 4) * 4;
    pl.segs = (pr.P + pl.segh - 1) / pl.segh;
    pl.kblocks = (pr.K + kKB - 1) / kKB;
    pl.cblocks = (pr.C + kCB - 1) / kCB;
    pl.units = pl.NB * pl.strips * pl.segs;
    const int blocks = pl.kblocks * pl.cblocks;
    int nsplit = (256 + blocks - 1) / blocks;
    if (nsplit > pl.units) nsplit = pl.units;
    if (nsplit < 1) nsplit = 1;
    pl.nsplit = nsplit;
    pl.part_bytes = nsplit > 1 ? (size_t)nsplit * pr.K * pr.C * 9 * sizeof(float) : 0;
    // small problems are not worth the two layout passes
    if ((size_t)pr.N * pr.P * pr.Q < 4096) return false;
    return true;
}

}  // namespace

bool bf16_wgrad_supports(const Problem& pr) {
    Plan pl;
    return make_plan(pr, pl);
}

size_t bf16_wgrad_workspace_bytes(const Problem& pr) {
    Plan pl;
    if (!make_plan(pr, pl)) return 0;
    return round256(pl.x_bytes) + round256(pl.y_bytes) + round256(pl.part_bytes);
}

hipError_t bf16_wgrad_run(const Problem& pr, const void* x, const void* dy, float* dw, void* ws, hipStream_t st) {
    Plan pl;
    if (!make_plan(pr, pl)) return hipErrorNotSupported;
    unsigned char* base = static_cast<unsigned char*>(ws);
    uint16_t* xP = reinterpret_cast<uint16_t*>(base);
    uint16_t* yP = reinterpret_cast<uint16_t*>(base + round256(pl.x_bytes));
    float* part = reinterpret_cast<float*>(base + round256(pl.x_bytes) + round256(pl.y_bytes));

    {
        PackNArgs a{static_cast<const uint16_t*>(x), xP, pr.N, pr.C, pr.H * pr.W,
                    (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * 2), pl.NB * pr.C * (pr.H * pr.W / 8)};
        pack_n8_kernel<<<(a.total + 255) / 256, 256, 0, st>>>(a);
        PackNArgs b{static_cast<const uint16_t*>(dy), yP, pr.N, pr.K, pr.P * pr.Q,
                    (unsigned)((size_t)pr.N * pr.K * pr.P * pr.Q * 2), pl.NB * pr.K * (pr.P * pr.Q / 8)};
        pack_n8_kernel<<<(b.total + 255) / 256, 256, 0, st>>>(b);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    BwArgs a{};
    a.xP = xP; a.dyP = yP; a.out = pl.nsplit > 1 ? part : dw;
    a.NB = pl.NB; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.K = pr.K; a.P = pr.P; a.Q = pr.Q;
    a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.strips = pl.strips; a.segs = pl.segs; a.segh = pl.segh;
    a.kblocks = pl.kblocks; a.cblocks = pl.cblocks; a.nsplit = pl.nsplit; a.units = pl.units;
    a.x_bytes = (unsigned)pl.x_bytes; a.y_bytes = (unsigned)pl.y_bytes;
    bf16_wgrad_kernel<<<pl.kblocks * pl.cblocks * pl.nsplit, 256, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1) return e;
    const size_t count = (size_t)pr.K * pr.C * 9;
    bf16_reduce_splits_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(part, dw, pl.nsplit, count);
    return hipGetLastError();
}

}  // namespace miconv
