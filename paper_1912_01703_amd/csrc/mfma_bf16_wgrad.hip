// Backward-weight 3x3 stride-1 convolution of bf16 tensors on the bf16 matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate, fp32 output), gfx950.
//
//   dw[k, c, r, s] = sum_{n, p, q} dy[n, k, p, q] * x[n, c, p - pad_h + r, q - pad_w + s]
//
// The reduction runs over images and pixels, and an MFMA lane supplies 8 consecutive reduction
// elements of its channel as one 16-byte register group.  If those 8 elements were neighbouring
// pixels, a tap shift of one pixel would misalign every x operand by 2 bytes.  They are therefore
// 8 images at the same pixel: LDS holds rows as [channel][column][8 images] (missing images are
// zeros), after which every tap shift is a multiple of 16 bytes and both operands are plain 16-byte
// LDS reads.  The transposition happens either on the way into LDS (8 narrow loads per 4 pixels and
// 16 byte-permutes; no extra memory) or in a pre-pass that rewrites x and dy into the caller's
// workspace as [N/8][channel][row][column][8 images] (copy speed, then 16-byte loads).  The first
// costs the main kernel about 70 % more time, the second one extra pass over x and dy: layers with
// few channels (little arithmetic per byte) take the first, the others the second.
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
// immediates; the only vector-ALU work in the MFMA loop are the byte-permutes of the in-kernel
// transposition.  Stores of the rows fetched during the previous stage and loads of the rows two
// stages ahead are spread between the MFMAs.
// Partial sums of the splits are added in split order by a second kernel: no float atomics.
#include "common.h"

#include <type_traits>

namespace miconv {
namespace {


// ---- pre-pass: [N][Ch][HW] -> [ceil(N/8)][Ch][HW][8] ------------------------------------------
struct PackNArgs {
    const uint16_t* src;
    uint16_t* dst;
    int N, Ch, HW;   // HW % 2 == 0 (planes start on 4-byte boundaries)
    unsigned src_bytes;
    int total;       // ceil(N/8) * Ch * ceil(HW / 8) threads
};

__global__ __launch_bounds__(256) void pack_n8_kernel(PackNArgs a) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= a.total) return;
    const int per = (a.HW + 7) / 8;   // the last group of a plane may run into the next plane: those pixels are not stored
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
    v4u v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)   // pixel j: its value in images 0..7
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const unsigned lo = r[2 * m][j / 2], hi = r[2 * m + 1][j / 2];
            v[j][m] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    if (8 * pc + 8 <= a.HW) {   // a whole group: eight stores in a row (per-store tests cost this kernel 70 % of its speed)
#pragma unroll
        for (int j = 0; j < 8; ++j) o[j] = v[j];
    } else {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            if (8 * pc + j < a.HW) o[j] = v[j];
    }
}

// ---- main kernel --------------------------------------------------------------------------------
struct BwArgs {
    const uint16_t* x;     // [N][C][H][W], or (PACKED) [NB][C][H][W][8]
    const uint16_t* dy;    // [N][K][P][Q], or (PACKED) [NB][K][P][Q][8]
    float* out;            // dw, or partial buffer [nsplit][K][C][9]
    int N, NB, C, H, W, K, P, Q;
    int pad_h, pad_w;
    int strips, segs, segh;    // unit = (image octet, strip, segment); segment height is a multiple of 4
    int kblocks, cblocks, nsplit, units;
};


constexpr int kSQ = 7, kSW = 4 * kSQ;                  // pixel groups and output columns per stage
constexpr int kXW = 32;                                // x columns kept per row: image columns q0-2 .. q0+29
constexpr int kKB = 64, kCB = 32;
constexpr int kDyRow = kSW * 16 + 16;                  // bytes per k in a dy row buffer (464: 20 banks mod 32)
constexpr int kDyBuf = kKB * kDyRow;
constexpr int kXRow = kXW * 16 + 16;                   // bytes per c in an x ring slot (528: 4 banks mod 32)
constexpr int kXSlot = kCB * kXRow;
constexpr int kDyBase = 4 * kXSlot;                    // the ring comes first: its slots are reachable by immediates
constexpr int kLds = kDyBase + 2 * kDyBuf;
static_assert((kCB * kXW / 4) % 256 == 0, "whole x groups per thread");
static_assert(3 * kXSlot + kXRow < 65536 && kDyBuf + kDyRow * 16 + kSW * 16 < 65536, "immediate offsets");

// Transposes four pixels of eight images: r[i] holds pixels 0..3 of image i as two dwords; the result
// for pixel j is one 16-byte group with the eight images in order.
__device__ __forceinline__ v4u gather_pixel(const v2u (&r)[8], int j) {
    v4u v;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
        const unsigned lo = r[2 * m][j / 2], hi = r[2 * m + 1][j / 2];
        v[m] = (j & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
    }
    return v;
}

// PACKED: x and dy come from the pre-pass (8 images innermost); otherwise they are transposed here.
template <bool PACKED>
__global__ __launch_bounds__(256) void bf16_wgrad_kernel(BwArgs a) {
    constexpr int SLOTS = kSQ * 9, RING = 9, PF = 6;
    static_assert(SLOTS % RING == 0 && PF < RING, "ring");
    __shared__ __attribute__((aligned(16))) unsigned char lds[kLds];

    // Workgroup ids that differ by multiples of 8 share an XCD (one L2 each).  Splits that follow each other work
    // on neighbouring strips of the same rows; they are given to one XCD, where they run side by side, so that a
    // cache line of a row, of which a 28-column strip covers 56 bytes, is fetched from HBM once and not once per strip
    // (3.2 GB of fetches for 0.8 GB of operands on 224x224 planes otherwise).
    const int blocks = a.kblocks * a.cblocks;
    const int wg = gridDim.x % 8 == 0 ? (int)(blockIdx.x % 8) * (int)(gridDim.x / 8) + (int)(blockIdx.x / 8) : (int)blockIdx.x;
    const int blk = wg % blocks, sp = wg / blocks;
    const int kb = blk / a.cblocks, cb = blk - kb * a.cblocks;
    const int k0 = kb * kKB, c0 = cb * kCB;
    const int u0 = __builtin_amdgcn_readfirstlane((int)((long long)a.units * sp / a.nsplit));
    const int u1 = __builtin_amdgcn_readfirstlane((int)((long long)a.units * (sp + 1) / a.nsplit));

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wk = wave & 1, wc = wave >> 1;
    const int li = lane & 15, g = lane >> 4;
    const int xplane = a.H * a.W, yplane = a.P * a.Q;

    // Gather plans.  Transposing: a thread owns NY groups of a dy row and NX of an x row; a group is
    // 4 neighbouring pixels of one channel in the 8 images of the unit.  PACKED: a thread owns single
    // pixels (16 bytes, neighbouring lanes neighbouring pixels).  Byte offsets are relative to (image,
    // first channel of the block, row 0, column 0); threads past the last dy item repeat an earlier one.
    constexpr unsigned EB = PACKED ? 16u : 2u;   // bytes per pixel of a channel row in global memory
    constexpr int YPX = PACKED ? 1 : 4;          // pixels per item
    constexpr int YPR = kSW / YPX, XPR = kXW / YPX;   // items per row
    constexpr int NY = (kKB * YPR + 255) / 256, NX = kCB * XPR / 256;   // items per thread
    unsigned ygo[NY];
    int ycol[NY];
    unsigned char* ysto[NY];
#pragma unroll
    for (int m = 0; m < NY; ++m) {
        const int e = (tid + 256 * m) % (kKB * YPR);
        const int kl = e / YPR, gq = e - kl * YPR;
        ygo[m] = k0 + kl < a.K ? (unsigned)(kl * yplane) * EB : kOob;   // the column is added per unit
        ycol[m] = YPX * gq;
        ysto[m] = lds + kDyBase + kl * kDyRow + YPX * gq * 16;
    }
    unsigned xgo[NX];
    int xcol[NX];
    unsigned char* xsto[NX];
#pragma unroll
    for (int m = 0; m < NX; ++m) {
        const int e = tid + 256 * m;
        const int cl = e / XPR, gx = e - cl * XPR;
        xgo[m] = c0 + cl < a.C ? (unsigned)(cl * xplane) * EB : kOob;   // the column is added per unit
        xcol[m] = YPX * gx - 2;
        xsto[m] = lds + cl * kXRow + YPX * gx * 16;
    }
    const unsigned char* ya = lds + kDyBase + (wk * 32 + li) * kDyRow + g * 16;
    // x column of pixel px and tap s: q0 + px + s - pad_w, kept at LDS column px + s + 2 - pad_w
    const unsigned char* xa = lds + (wc * 16 + li) * kXRow + (g + 2 - a.pad_w) * 16;

    v4f acc[2][9];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int t = 0; t < 9; ++t) acc[i][t] = v4f{0.f, 0.f, 0.f, 0.f};

    const int nimg = PACKED ? a.NB : a.N;   // images, or octets of images, in the tensors
    const rsrc_t yrs = make_rsrc(a.dy, (unsigned)((size_t)nimg * a.K * yplane * EB)), xrs = make_rsrc(a.x, (unsigned)((size_t)nimg * a.C * xplane * EB));
    const rsrc_t nors = make_rsrc(a.dy, 0);
    v2u yreg[PACKED ? 1 : NY][8];         // [group][image]
    unsigned xreg[PACKED ? 1 : NX][8][2];   // [group][image][pixel pair]: the pairs are loaded (and bounds-checked) separately
    v4u yreg4[PACKED ? NY : 1], xreg4[PACKED ? NX : 1];   // PACKED: [pixel], already 8 images each
    v4u ring[RING], A[2][2];

    for (int unit = u0; unit < u1; ++unit) {
        int u = unit;
        const int seg = __builtin_amdgcn_readfirstlane(u % a.segs); u /= a.segs;
        const int strip = __builtin_amdgcn_readfirstlane(u % a.strips);
        const int nb = __builtin_amdgcn_readfirstlane(u / a.strips);
        const int q0 = strip * kSW;
        const int ps = seg * a.segh, pe = ps + a.segh < a.P ? ps + a.segh : a.P;
        // per-lane column validity of this strip (transposing: Q is a multiple of 4 and W is even, so
        // groups of dy and pixel pairs of x are valid or invalid as a whole)
        constexpr int XD = PACKED ? 1 : 2;
        unsigned yv[NY], xv[NX][XD];
#pragma unroll
        for (int m = 0; m < NY; ++m) yv[m] = q0 + ycol[m] < a.Q ? ygo[m] + (unsigned)(q0 + ycol[m]) * EB : kOob;
#pragma unroll
        for (int m = 0; m < NX; ++m)
#pragma unroll
            for (int d = 0; d < XD; ++d) {
                const int col = q0 + xcol[m] + 2 * d;
                xv[m][d] = col >= 0 && col < a.W && xgo[m] != kOob ? xgo[m] + (unsigned)col * EB : kOob;
            }
        const int n0 = nb * 8;

        // Stage p: store the rows fetched during stage p-1 (dy row p+1, x row p+3-pad_h), multiply output
        // row p, fetch dy row p+2 and x row p+4-pad_h.  The four stages before the first row only fill LDS.
        auto stage = [&](auto phc, auto fillc, int p) __attribute__((always_inline)) {
            constexpr int PH4 = decltype(phc)::value;            // p mod 4
            constexpr bool FILL = decltype(fillc)::value;        // a stage before the first row: no arithmetic
            constexpr int YB = (PH4 & 1) * kDyBuf;               // dy buffer multiplied in this stage
            constexpr int YW = ((PH4 + 1) & 1) * kDyBuf;         // ... and stored to
            constexpr int XWS = ((PH4 + 3) & 3) * kXSlot;        // ring slot stored to
            const int yr = p + 2, xr = p + 4 - a.pad_h;          // rows fetched in this stage
            const bool yok = yr >= ps && yr < pe, xok = xr >= 0 && xr < a.H;
            // one piece = one pixel: stored as loaded, or transposed out of the held group registers
            auto store_piece = [&](int pi) __attribute__((always_inline)) {
                if constexpr (PACKED) {
                    if (pi < NY) *reinterpret_cast<v4u*>(ysto[pi] + YW) = yreg4[pi];
                    else *reinterpret_cast<v4u*>(xsto[pi - NY] + XWS) = xreg4[pi - NY];
                } else {
                    const int grp = pi / 4, j = pi % 4;
                    if (grp < NY) {
                        *reinterpret_cast<v4u*>(ysto[grp] + YW + j * 16) = gather_pixel(yreg[grp], j);
                    } else {
                        const int m = grp - NY;
                        v2u r[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) r[i] = v2u{xreg[m][i][0], xreg[m][i][1]};
                        *reinterpret_cast<v4u*>(xsto[m] + XWS + j * 16) = gather_pixel(r, j);
                    }
                }
            };
            // Load step i: one pixel (PACKED), or image i of the octet for every group.  The per-lane offset
            // addresses (channel, column); image or octet, first channel and row go into the scalar offset;
            // an absent image or row reads zeros.
            const unsigned yrow = (unsigned)(k0 * yplane + yr * a.Q) * EB, xrow = (unsigned)(c0 * xplane + xr * a.W) * EB;
            const unsigned yimg = (unsigned)(a.K * yplane) * EB, ximg = (unsigned)(a.C * xplane) * EB;
            constexpr int NPIECE = PACKED ? NY + NX : 4 * (NY + NX);
            constexpr int NLOAD = PACKED ? NY + NX : 8, LSTEP = PACKED ? 3 : 4;
            auto load_step = [&](int i) __attribute__((always_inline)) {
                if constexpr (PACKED) {
                    if (i < NY)
                        yreg4[i] = __builtin_amdgcn_raw_buffer_load_b128(yok ? yrs : nors, yv[i], yok ? (unsigned)nb * yimg + yrow : 0u, 0);
                    else
                        xreg4[i - NY] = __builtin_amdgcn_raw_buffer_load_b128(xok ? xrs : nors, xv[i - NY][0], xok ? (unsigned)nb * ximg + xrow : 0u, 0);
                } else {
                    const bool have = n0 + i < a.N;
                    const rsrc_t yd = have && yok ? yrs : nors, xd = have && xok ? xrs : nors;
                    const unsigned ys = have && yok ? (unsigned)(n0 + i) * yimg + yrow : 0u;
                    const unsigned xso = have && xok ? (unsigned)(n0 + i) * ximg + xrow : 0u;
#pragma unroll
                    for (int m = 0; m < NY; ++m) yreg[m][i] = __builtin_amdgcn_raw_buffer_load_b64(yd, yv[m], ys, 0);
#pragma unroll
                    for (int m = 0; m < NX; ++m)
#pragma unroll
                        for (int d = 0; d < 2; ++d) xreg[m][i][d] = __builtin_amdgcn_raw_buffer_load_b32(xd, xv[m][d], xso, 0);
                }
            };
            constexpr int LB = 2 * NPIECE + 2;   // first load slot
            static_assert(LB + LSTEP * (NLOAD - 1) < SLOTS, "stores, then loads, inside one stage");
            __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): the held rows were requested a stage ago
            if constexpr (!FILL) {
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
                    // rows for the next stage: registers -> (transposed) -> LDS in the first 24 slots, then the
                    // same registers are refilled, image by image, with the rows for the stage after it
                    if (s % 2 == 0 && s / 2 < NPIECE) store_piece(s / 2);
                    if (s >= LB && (s - LB) % LSTEP == 0 && (s - LB) / LSTEP < NLOAD) load_step((s - LB) / LSTEP);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
#pragma unroll
                for (int pi = 0; pi < NPIECE; ++pi) store_piece(pi);
#pragma unroll
                for (int i = 0; i < NLOAD; ++i) load_step(i);
            }
            __syncthreads();
        };

        // before the unit's first stage the registers must hold defined values (they are stored, unused)
        if constexpr (PACKED) {
#pragma unroll
            for (int m = 0; m < NY; ++m) yreg4[m] = v4u{0, 0, 0, 0};
#pragma unroll
            for (int m = 0; m < NX; ++m) xreg4[m] = v4u{0, 0, 0, 0};
        } else {
#pragma unroll
            for (int m = 0; m < NY; ++m)
#pragma unroll
                for (int i = 0; i < 8; ++i) yreg[m][i] = v2u{0, 0};
#pragma unroll
            for (int m = 0; m < NX; ++m)
#pragma unroll
                for (int i = 0; i < 8; ++i) xreg[m][i][0] = xreg[m][i][1] = 0;
        }
        __syncthreads();   // the previous unit's last reads are done before its rows are overwritten
        using std::integral_constant;
        // ps is a multiple of 4: the four stages before it fill LDS, then the row loop is free of branches
        // that would make the accumulators change registers
        stage(integral_constant<int, 0>{}, std::true_type{}, ps - 4);
        stage(integral_constant<int, 1>{}, std::true_type{}, ps - 3);
        stage(integral_constant<int, 2>{}, std::true_type{}, ps - 2);
        stage(integral_constant<int, 3>{}, std::true_type{}, ps - 1);
        for (int p = ps; p < pe; p += 4) {
            stage(integral_constant<int, 0>{}, std::false_type{}, p);
            if (p + 1 >= pe) break;
            stage(integral_constant<int, 1>{}, std::false_type{}, p + 1);
            if (p + 2 >= pe) break;
            stage(integral_constant<int, 2>{}, std::false_type{}, p + 2);
            if (p + 3 >= pe) break;
            stage(integral_constant<int, 3>{}, std::false_type{}, p + 3);
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

// Sums the partial buffers in a fixed order, one thread per element.
__global__ __launch_bounds__(256) void bf16_reduce_few_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                     int nsplit, size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = part[i];
    for (int s = 1; s < nsplit; ++s) sum += part[(size_t)s * count + i];
    dw[i] = sum;
}

// The same with few elements and many splits (64 x 64 channels: 36 864 elements, 128 splits), where one thread per
// element leaves most of the machine idle behind 128 loads in a row (31 us): eight threads share an element, each adds
// every eighth split, and the eight sums meet in LDS in thread order.
__global__ __launch_bounds__(256) void bf16_reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw,
                                                                 int nsplit, size_t count) {
    __shared__ float red[8][32];
    const int e = threadIdx.x & 31, g = threadIdx.x >> 5;
    const size_t i = (size_t)blockIdx.x * 32 + e;
    float sum = 0.f;
    if (i < count)
        for (int s = g; s < nsplit; s += 8) sum += part[(size_t)s * count + i];
    red[g][e] = sum;
    __syncthreads();
    if (g == 0 && i < count) {
        float total = red[0][e];
#pragma unroll
        for (int k = 1; k < 8; ++k) total += red[k][e];
        dw[i] = total;
    }
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

struct Plan {
    int NB, strips, segs, segh, kblocks, cblocks, nsplit, units;
    bool packed;                         // operands rewritten by the pre-pass
    size_t x_bytes, y_bytes, part_bytes; // workspace: packed x, packed dy (0 unless packed), partial sums
};

bool make_plan(const Problem& pr, Plan& pl) {
    if (pr.dtype != 1 || pr.R != 3 || pr.S != 3 || pr.sh != 1 || pr.sw != 1 || pr.groups != 1) return false;
    if (pr.ph > 2 || pr.pw > 2) return false;
    const size_t lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * pr.H * pr.W * 2 >= lim || (size_t)pr.N * pr.K * pr.P * pr.Q * 2 >= lim) return false;
    pl.NB = (pr.N + 7) / 8;
    // The pre-pass moves 4 bytes per element of x and dy at copy speed; transposing in the main kernel
    // slows that kernel by about 0.7x its 18 K C flops per pixel at ~1 PFLOP/s.  The two cost the same
    // near K C / (K + C) = 60.
    pl.x_bytes = (size_t)pl.NB * pr.C * pr.H * pr.W * 16;
    pl.y_bytes = (size_t)pl.NB * pr.K * pr.P * pr.Q * 16;
    pl.packed = (size_t)pr.K * pr.C >= (size_t)60 * (pr.K + pr.C) && (pr.H * pr.W) % 2 == 0 && (pr.P * pr.Q) % 2 == 0 &&
                pl.x_bytes < lim && pl.y_bytes < lim;
    if (!pl.packed) {
        pl.x_bytes = pl.y_bytes = 0;
        if (pr.Q % 4 != 0 || pr.W % 2 != 0) return false;   // groups of 4 dy pixels and pairs of x pixels never straddle a row end
    }
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
    // small problems gain nothing over the fp32 kernels
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
    // every load here is 4 bytes or wider: tensors that start on an odd element go to the kernels that take any alignment
    if (reinterpret_cast<uintptr_t>(x) % 4 != 0 || reinterpret_cast<uintptr_t>(dy) % 4 != 0) return hipErrorNotSupported;
    unsigned char* base = static_cast<unsigned char*>(ws);
    uint16_t* xP = reinterpret_cast<uint16_t*>(base);
    uint16_t* yP = reinterpret_cast<uint16_t*>(base + round256(pl.x_bytes));
    float* part = reinterpret_cast<float*>(base + round256(pl.x_bytes) + round256(pl.y_bytes));

    BwArgs a{};
    a.x = static_cast<const uint16_t*>(x); a.dy = static_cast<const uint16_t*>(dy);
    if (pl.packed) {
        PackNArgs px{a.x, xP, pr.N, pr.C, pr.H * pr.W, (unsigned)((size_t)pr.N * pr.C * pr.H * pr.W * 2),
                     pl.NB * pr.C * ((pr.H * pr.W + 7) / 8)};
        pack_n8_kernel<<<(px.total + 255) / 256, 256, 0, st>>>(px);
        PackNArgs py{a.dy, yP, pr.N, pr.K, pr.P * pr.Q, (unsigned)((size_t)pr.N * pr.K * pr.P * pr.Q * 2),
                     pl.NB * pr.K * ((pr.P * pr.Q + 7) / 8)};
        pack_n8_kernel<<<(py.total + 255) / 256, 256, 0, st>>>(py);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        a.x = xP; a.dy = yP;
    }
    a.out = pl.nsplit > 1 ? part : dw;
    a.N = pr.N; a.NB = pl.NB; a.C = pr.C; a.H = pr.H; a.W = pr.W; a.K = pr.K; a.P = pr.P; a.Q = pr.Q;
    a.pad_h = pr.ph; a.pad_w = pr.pw;
    a.strips = pl.strips; a.segs = pl.segs; a.segh = pl.segh;
    a.kblocks = pl.kblocks; a.cblocks = pl.cblocks; a.nsplit = pl.nsplit; a.units = pl.units;
    const unsigned grid = (unsigned)(pl.kblocks * pl.cblocks * pl.nsplit);
    if (pl.packed) bf16_wgrad_kernel<true><<<grid, 256, 0, st>>>(a);
    else bf16_wgrad_kernel<false><<<grid, 256, 0, st>>>(a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || pl.nsplit == 1) return e;
    const size_t count = (size_t)pr.K * pr.C * 9;
    if (pl.nsplit >= 16) bf16_reduce_splits_kernel<<<(unsigned)((count + 31) / 32), 256, 0, st>>>(part, dw, pl.nsplit, count);
    else bf16_reduce_few_splits_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(part, dw, pl.nsplit, count);
    return hipGetLastError();
}

}  // namespace miconv
