// 1x1 convolutions (stride 1, no padding, one group) of bf16 tensors on the bf16 matrix cores
// (v_mfma_f32_16x16x32_bf16, fp32 accumulate), gfx950.  A 1x1 convolution is a matrix product, and all three passes
// are the same kernel, C[m][n] = sum_k A[m][k] * B[n][k], with both operands contiguous along k:
//
//   forward        y [img][f][hw] = sum_c w[f][c]  * xT [img*HW+hw][c]     A = w,            B = x  channels-innermost
//   backward-data  dx[img][c][hw] = sum_k wT[c][k] * dyT[img*HW+hw][k]     A = w transposed, B = dy channels-innermost
//   backward-weight dw[k][c] = sum_img sum_hw dy[img][k][hw] * x[img][c][hw]   A = dy, B = x as they are (NCHW rows are
//                                                                          contiguous along hw), one "batch" per image
//
// The channels-innermost copies (and the transposed filter) are made by small pre-passes into the caller's workspace.
// A workgroup of four waves owns a 64 x 64 tile of C and walks k in chunks of 64: the A and B tiles of a chunk go
// from global memory (16 bytes per lane, rows of 128 bytes) through registers into one of two LDS buffers while the
// other buffer is multiplied; a wave owns a quarter of the tile (2 x 2 MFMA blocks per 32 elements of k).
// Backward-weight splits the images over the workgroups of a tile and a second kernel adds the partial results in
// split order (no atomics: bit-reproducible).  Rows shorter than a chunk's reach read zeros: offsets beyond a row's
// end are given the out-of-range marker, and the one 16-byte piece that straddles the end of a row whose length is
// no multiple of 8 has its surplus elements cleared before it is stored to LDS.
#include "common.h"
#include <type_traits>

namespace miconv {
namespace {

constexpr int BK = 64;                           // elements of k per chunk
constexpr int PITCH = BK * 2 + 16;               // bytes per tile row in LDS: 8 consecutive rows hit distinct banks
constexpr int NTHREADS = 256;

struct GemmArgs {
    const uint16_t* A;
    const uint16_t* B;
    void* out;                 // mode 0: [img][M][HW] (float or bf16); mode 1: float [split][M][N]
    int M, N, Kd;              // rows of A, rows of B, reduction length per batch
    int lda, ldb;              // elements between rows
    long long a_batch, b_batch;   // elements between batches
    int batches, splits;       // reduction batches, and how many workgroups share a tile's batches
    int tiles_m, tiles_n;
    int mode, HW, out_bf16;
    // fused epilogues of mode 0 (both null: none): y = max(0, y + bias[m]); dx = mask > 0 ? dx : 0 (mask: bf16, shaped like out)
    const float* bias;
    const uint16_t* mask;
};

__device__ __forceinline__ unsigned pack_bf16_pair(float lo, float hi) {
    const unsigned a = __float_as_uint(lo), b = __float_as_uint(hi);
    return ((a + 0x7FFFu + ((a >> 16) & 1u)) >> 16) | ((b + 0x7FFFu + ((b >> 16) & 1u)) & 0xFFFF0000u);
}

// BM x BN: the workgroup's tile of C (multiples of 32; a wave owns a quarter, BM/2 x BN/2).  Large tiles read each
// operand byte from LDS less often; small tiles put more workgroups on a CU, and it is the other workgroups' MFMAs that
// cover the time a chunk's loads take to arrive (a chunk is multiplied in a few hundred cycles, a load takes thousands).
// DEPTH: chunks kept in flight in registers (1 or 2).  With two register sets a chunk's loads are issued two chunks
// of MFMAs before they are needed instead of one.
// BT: B is not given with k innermost but as an NCHW tensor [img][k][HW] whose rows n = img * HW + hw are its pixels
// (forward: x, backward-data: dy), and is transposed on the way into LDS: half of the threads each fetch, for eight
// channel planes, the same aligned group of four pixels (eight 8-byte loads, the plane picked by the scalar offset;
// lanes run along the pixels), and byte permutes turn the 8 x 4 values into the four 16-byte pieces "eight channels of
// one pixel".  Planes are multiples of four pixels, so a group never straddles two images.  This saves writing and
// re-reading a channels-innermost copy of the tensor (17 of 54 us on 512 -> 512 channels at 14 x 14, N = 128).
template <int BM, int BN, int OCC, int DEPTH, bool BT>
__global__ __launch_bounds__(NTHREADS, OCC) void bf16_gemm_kernel(GemmArgs a) {
    static_assert(!BT || (BN == 64 && BK == 64), "the in-flight transposition is laid out for 64 pixels x 64 channels");
    constexpr int MB = BM / 32, NB = BN / 32;                  // 16 x 16 blocks per wave along m and n
    constexpr int PA = BM * (BK / 8) / NTHREADS, PB = BN * (BK / 8) / NTHREADS;   // 16-byte pieces per thread
    constexpr int A_BYTES = BM * PITCH, BUF_BYTES = (BM + BN) * PITCH;
    __shared__ __attribute__((aligned(16))) unsigned char lds[2 * BUF_BYTES];   // [buffer][A | B]
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave & 1, wn = wave >> 1;
    const int li = lane & 15, kk = lane >> 4;
    // workgroup -> (tile, split): the tiles of one split are neighbours, m fastest.  Consecutive workgroup ids land on
    // different XCDs (8, one L2 each): every XCD is given a contiguous run of the tile sequence, so that the workgroups
    // which share a B tile (the m tiles of one n tile) share an L2 and run at about the same time; dealt round-robin,
    // every L2 fetched every B tile itself.
    const int tiles = a.tiles_m * a.tiles_n;
    const int per_xcd = (tiles * a.splits + 7) >> 3;
    const int wg = ((int)blockIdx.x & 7) * per_xcd + ((int)blockIdx.x >> 3);
    if (((int)blockIdx.x >> 3) >= per_xcd || wg >= tiles * a.splits) return;   // the whole workgroup: no barrier is missed
    const int tile = wg % tiles, sp = wg / tiles;
    const int m0 = (tile % a.tiles_m) * BM, n0 = (tile / a.tiles_m) * BN;
    const int b_begin = (int)((long long)a.batches * sp / a.splits), b_end = (int)((long long)a.batches * (sp + 1) / a.splits);
    const int chunks = (a.Kd + BK - 1) / BK;
    const int total = (b_end - b_begin) * chunks;

    // this thread's pieces of a tile: row r = p / 8, elements 8 * (p % 8) .. + 7 of the chunk
    constexpr int PMAX = PA > PB ? PA : PB;
    int prow[PMAX], plds[PMAX];
    const int pcol = (tid & 7) * 8;
#pragma unroll
    for (int i = 0; i < PMAX; ++i) {
        const int p = tid + NTHREADS * i;
        prow[i] = p >> 3;
        plds[i] = prow[i] * PITCH + pcol * 2;
    }
    const bool ktail = (a.Kd & 7) != 0;

    v4u ra[DEPTH][PA], rb[DEPTH][BT ? 1 : PB];
    v2u rt[DEPTH][BT ? 8 : 1];   // BT: four pixels of eight channel planes
    int nva[DEPTH];   // elements of this thread's pieces inside their rows (for the piece that straddles a row's end)
    // Row offsets are fixed for the whole kernel (rows past the tile's operand: the out-of-range marker, which stays
    // out of range when a chunk's offset, below 2^31, is added); the chunk walk keeps its batch and k position in counters, so a
    // fetch is a handful of scalar operations and one add per load.
    unsigned aoff[PA], boff[PB];
#pragma unroll
    for (int i = 0; i < PA; ++i) aoff[i] = m0 + prow[i] < a.M ? (unsigned)((m0 + prow[i]) * a.lda + pcol) * 2u : kOob;
#pragma unroll
    for (int i = 0; i < PB; ++i) boff[i] = n0 + prow[i] < a.N ? (unsigned)((n0 + prow[i]) * a.ldb + pcol) * 2u : kOob;
    const unsigned a_bytes = (unsigned)((size_t)a.M * a.lda * 2);
    const unsigned b_bytes = BT ? (unsigned)((size_t)a.N * a.Kd * 2) : (unsigned)((size_t)a.N * a.ldb * 2);
    // BT: thread u < 128 owns pixel group u % 16 (pixels n0 + 4 * (u % 16) ..) and channel group u / 16 of a chunk
    const int tpg = tid & 15, tcg = tid >> 4;
    unsigned toff = kOob;                 // byte offset of (image, channel 8 * tcg, pixel) or the out-of-range marker
    int tlds = 0;
    if constexpr (BT) {
        const int n = n0 + 4 * tpg;
        if (tid < 128 && n < a.N) {
            const int img = n / a.HW, hw = n - img * a.HW;
            toff = (unsigned)((img * a.Kd + 8 * tcg) * a.HW + hw) * 2u;
        }
        tlds = 4 * tpg * PITCH + tcg * 16;
    }
    const unsigned plane_bytes = (unsigned)a.HW * 2u;
    int fb = b_begin, fk = 0;   // batch and first k of the next chunk to fetch
    // the descriptors change with the batch only (once per image in backward-weight, never otherwise)
    rsrc_t ars = make_rsrc(a.A + (size_t)fb * a.a_batch, a_bytes);
    rsrc_t brs = make_rsrc(a.B + (size_t)fb * a.b_batch, b_bytes);
    auto fetch = [&](auto setc) __attribute__((always_inline)) {
        constexpr int SET = decltype(setc)::value;
        const bool kin = fk + pcol < a.Kd;   // else this thread's pieces lie beyond their rows: zeros
        const unsigned kb = (unsigned)fk * 2u;
#pragma unroll
        for (int i = 0; i < PA; ++i) ra[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(ars, kin ? aoff[i] + kb : kOob, 0, 0);
        if constexpr (BT) {
            // (a valid group has its eight planes inside the tensor; channels past the last chunk's end: out of range)
            const unsigned off = fk + 8 * tcg < a.Kd ? toff + (unsigned)fk * plane_bytes : kOob;
#pragma unroll
            for (int j = 0; j < 8; ++j) rt[SET][j] = __builtin_amdgcn_raw_buffer_load_b64(brs, off, j * plane_bytes, 0);
        } else {
#pragma unroll
            for (int i = 0; i < PB; ++i) rb[SET][i] = __builtin_amdgcn_raw_buffer_load_b128(brs, kin ? boff[i] + kb : kOob, 0, 0);
        }
        nva[SET] = a.Kd - (fk + pcol);
        fk += BK;
        if (fk >= a.Kd) {
            fk = 0;
            ++fb;
            ars = make_rsrc(a.A + (size_t)fb * a.a_batch, a_bytes);
            brs = make_rsrc(a.B + (size_t)fb * a.b_batch, b_bytes);
        }
    };
    auto stash = [&](int buf, auto setc) __attribute__((always_inline)) {
        constexpr int SET = decltype(setc)::value;
        unsigned char* la = lds + buf * BUF_BYTES;
        unsigned char* lb = la + A_BYTES;
        auto put = [&](unsigned char* dst, v4u v) __attribute__((always_inline)) {
            if (ktail) {   // (row lengths are even: whole dwords)
#pragma unroll
                for (int d = 0; d < 4; ++d) v[d] = 2 * d < nva[SET] ? v[d] : 0u;
            }
            *reinterpret_cast<v4u*>(dst) = v;
        };
#pragma unroll
        for (int i = 0; i < PA; ++i) put(la + plds[i], ra[SET][i]);
        if constexpr (BT) {
            if (tid < 128) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {   // pixel k of the group: channels 2i, 2i+1 are the halves k % 2 of dword k / 2 of planes 2i, 2i+1
                    v4u piece;
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        piece[i] = __builtin_amdgcn_perm(rt[SET][2 * i + 1][k / 2], rt[SET][2 * i][k / 2], k % 2 ? 0x07060302u : 0x05040100u);
                    *reinterpret_cast<v4u*>(lb + tlds + k * PITCH) = piece;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < PB; ++i) put(lb + plds[i], rb[SET][i]);
        }
    };

    v4f acc[MB][NB];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = v4f{0.f, 0.f, 0.f, 0.f};

    using S0 = std::integral_constant<int, 0>;
    using S1 = std::integral_constant<int, DEPTH - 1>;
    // chunk 0 goes to LDS; chunks 1 .. DEPTH wait in the register sets (chunk c in set (c - 1) % DEPTH)
    if (total > 0) {
        fetch(S0{});
        stash(0, S0{});
    }
    if (total > 1) fetch(S0{});
    if (DEPTH == 2 && total > 2) fetch(S1{});
    __syncthreads();
    // operand addresses of this lane: row (wave's 64-row share + 16 * block + li), 16 bytes at k = 8 * kk of a k-step
    const int arow = (wm * (BM / 2) + li) * PITCH + kk * 16, brow = (wn * (BN / 2) + li) * PITCH + kk * 16;
    auto multiply = [&](int t) __attribute__((always_inline)) {
        const unsigned char* la = lds + (t & 1) * BUF_BYTES;
        const unsigned char* lb = la + A_BYTES;
#pragma unroll
        for (int ks = 0; ks < BK / 32; ++ks) {
            v4u fa[MB], fb[NB];
#pragma unroll
            for (int i = 0; i < MB; ++i) fa[i] = *reinterpret_cast<const v4u*>(la + arow + i * 16 * PITCH + ks * 64);
#pragma unroll
            for (int j = 0; j < NB; ++j) fb[j] = *reinterpret_cast<const v4u*>(lb + brow + j * 16 * PITCH + ks * 64);
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int j = 0; j < NB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(v8bf, fa[i]), __builtin_bit_cast(v8bf, fb[j]),
                                                                        acc[i][j], 0, 0, 0);
        }
    };
    // iteration t: multiply chunk t, move chunk t + 1 from its register set to the other LDS buffer, refill that set
    // with chunk t + 1 + DEPTH
    for (int t = 0; t < total; t += DEPTH) {
        multiply(t);
        if (t + 1 < total) stash((t + 1) & 1, S0{});
        if (t + 1 + DEPTH < total) fetch(S0{});
        __syncthreads();
        if (DEPTH == 2 && t + 1 < total) {
            multiply(t + 1);
            if (t + 2 < total) stash(t & 1, S1{});
            if (t + 4 < total) fetch(S1{});
            __syncthreads();
        }
    }

    // ---- write-out: D[m = 4 * kk + v][n = li] of block (i, j) ---------------------------------------------------
#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int n = n0 + wn * (BN / 2) + j * 16 + li;
        if (n >= a.N) continue;
        size_t nbase;      // offset of (m = 0, n), and the distance between consecutive m
        size_t mstride;
        if (a.mode == 0) {
            const int img = n / a.HW, hw = n - img * a.HW;
            nbase = (size_t)img * a.M * a.HW + hw;
            mstride = (size_t)a.HW;
        } else {
            nbase = (size_t)sp * a.M * a.N + n;
            mstride = (size_t)a.N;
        }
        if (a.bias) {   // (wave-uniform branches on kernel arguments)
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = m0 + wm * (BM / 2) + i * 16 + 4 * kk + v;
                    acc[i][j][v] = fmaxf(acc[i][j][v] + (m < a.M ? a.bias[m] : 0.f), 0.f);
                }
        }
        if (a.mask) {   // the mask elements under this column's results are requested together, then applied
            float mv[MB][4];
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const int m = m0 + wm * (BM / 2) + i * 16 + 4 * kk + v;
                    mv[i][v] = m < a.M ? bf16_to_float(a.mask[nbase + (size_t)m * mstride]) : 0.f;
                }
#pragma unroll
            for (int i = 0; i < MB; ++i)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[i][j][v] = mv[i][v] > 0.f ? acc[i][j][v] : 0.f;
        }
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int m = m0 + wm * (BM / 2) + i * 16 + 4 * kk + v;
                if (m >= a.M) continue;
                const size_t e = nbase + (size_t)m * mstride;
                if (a.out_bf16) static_cast<uint16_t*>(a.out)[e] = static_cast<uint16_t>(pack_bf16_pair(acc[i][j][v], 0.f));
                else static_cast<float*>(a.out)[e] = acc[i][j][v];
            }
    }
}

// [N][Ch][HW] -> [N][HW][Ch]: a workgroup moves 128 pixels x 64 channels through LDS: 16-byte loads along the pixels
// (lanes along a channel row), 16-byte stores along the channels (8 lanes write the 128 contiguous bytes of a pixel's
// 64 channels, a wave whole cache lines).  Ch is a multiple of 8, planes have an even number of pixels.
struct PackArgs {
    const uint16_t* src;
    uint16_t* dst;
    int N, Ch, HW;
    unsigned src_bytes;
};
__global__ __launch_bounds__(256) void gemm_pack_nhwc_kernel(PackArgs a) {
    constexpr int TP = 128, LS = TP + 8;   // pixels per tile; elements per LDS row (16-byte aligned rows)
    __shared__ __attribute__((aligned(16))) uint16_t tile[64 * LS];   // [channel][pixel]
    const int t = threadIdx.x;
    const int p0 = blockIdx.x * TP, c0 = blockIdx.y * 64, n = blockIdx.z;
    const rsrc_t rs = make_rsrc(a.src, a.src_bytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = t + 256 * i;
        const int c = q >> 4, pc = q & 15;   // 8 pixels of channel c; a group that runs past the plane picks up values nobody reads
        const int p = p0 + 8 * pc;
        const unsigned off = p < a.HW && c0 + c < a.Ch ? (unsigned)((n * a.Ch + c0 + c) * a.HW + p) * 2u : kOob;
        *reinterpret_cast<v4u*>(&tile[c * LS + 8 * pc]) = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
    }
    __syncthreads();
    const int g = t & 7;   // this thread's 8 channels: a group exists as a whole or not at all
    if (c0 + 8 * g >= a.Ch) return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int px = (t >> 3) + 32 * i, p = p0 + px;
        if (p >= a.HW) continue;
        v4u o;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            o[j] = (unsigned)tile[(8 * g + 2 * j) * LS + px] | ((unsigned)tile[(8 * g + 2 * j + 1) * LS + px] << 16);
        *reinterpret_cast<v4u*>(a.dst + ((size_t)n * a.HW + p) * a.Ch + c0 + 8 * g) = o;
    }
}

// w[K][C] -> wT[C][K]
__global__ __launch_bounds__(256) void gemm_transpose_kernel(const uint16_t* __restrict__ w, uint16_t* __restrict__ wt, int K, int C) {
    __shared__ uint16_t tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    const int c0 = blockIdx.x * 32, k0 = blockIdx.y * 32;
    for (int r = ty; r < 32; r += 8)
        if (k0 + r < K && c0 + tx < C) tile[r][tx] = w[(size_t)(k0 + r) * C + c0 + tx];
    __syncthreads();
    for (int r = ty; r < 32; r += 8)
        if (c0 + r < C && k0 + tx < K) wt[(size_t)(c0 + r) * K + k0 + tx] = tile[tx][r];
}

__global__ __launch_bounds__(256) void gemm_reduce_splits_kernel(const float* __restrict__ part, float* __restrict__ dw, int nsplit,
                                                                 size_t count) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= count) return;
    float sum = part[i];
    for (int s = 1; s < nsplit; ++s) sum += part[(size_t)s * count + i];
    dw[i] = sum;
}

size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

bool shape_ok(int pass, const Problem& pr) {
    if (pr.dtype != 1 || pr.R != 1 || pr.S != 1 || pr.sh != 1 || pr.sw != 1 || pr.ph != 0 || pr.pw != 0 || pr.groups != 1) return false;
    const long long HW = (long long)pr.H * pr.W;
    if (HW % 2 != 0) return false;                    // rows of the NCHW tensors start on 4-byte boundaries
    if (pr.C % 8 != 0 || pr.K % 8 != 0) return false; // rows of the channels-innermost copies and of the filter start on 16-byte boundaries
    const size_t lim = (size_t)1 << 31;
    if ((size_t)pr.N * pr.C * HW * 2 >= lim || (size_t)pr.N * pr.K * HW * 2 >= lim || (size_t)pr.K * pr.C * 2 >= lim) return false;
    if ((size_t)pr.N * HW * (pass == 0 ? pr.K : pr.C) * 4 >= ((size_t)1 << 33)) return false;
    // small problems gain nothing over the fp32 kernels
    return (size_t)pr.N * HW * pr.C * pr.K >= ((size_t)1 << 24);
}

// Tile edge.  64 x 64 tiles with four workgroups per CU beat 128 x 128 tiles with two on both 1x1 benchmark layers
// (1024 -> 256 channels at 14 x 14, N = 64: 41 against 55 us forward; 512 -> 512, N = 128: 54 against 66 us): with the
// larger tile a workgroup waits for its chunk's loads and too few others are there to fill the time.
constexpr int kEdge = 64;

// Backward-weight: the images are split so that about 1024 workgroups (four per CU) share the work.
int wgrad_splits(const Problem& pr) {
    const int tiles = ((pr.K + kEdge - 1) / kEdge) * ((pr.C + kEdge - 1) / kEdge);
    int s = (1024 + tiles - 1) / tiles;
    if (s > pr.N) s = pr.N;
    return s < 1 ? 1 : s;
}

}  // namespace

bool bf16_gemm_supports(int pass, const Problem& pr) { return pass >= 0 && pass <= 2 && shape_ok(pass, pr); }

bool bf16_gemm_accepts(int pass, const Problem& pr, const void* in0, const void* in1) {
    return bf16_gemm_supports(pass, pr) && reinterpret_cast<uintptr_t>(in0) % 4 == 0 && reinterpret_cast<uintptr_t>(in1) % 4 == 0;
}

// Planes of a multiple of four pixels can be transposed inside the product kernel instead of getting a channels-
// innermost copy.  Every m tile of a pixel tile then transposes the same B data again (with 8-byte loads on half of the
// threads), so this pays only with few destination channels: 1024 -> 256 channels forward 40 -> 33 us (4 m tiles), but
// 512 -> 512 54 -> 56 us (8) and 256 -> 1024 backward-data 36 -> 41 us (16).
bool transposes_in_flight(int pass, const Problem& pr) {
    return ((long long)pr.H * pr.W) % 4 == 0 && (pass == 0 ? pr.K : pr.C) <= 4 * kEdge;
}

size_t bf16_gemm_workspace_bytes(int pass, const Problem& pr) {
    if (!bf16_gemm_supports(pass, pr)) return 0;
    const size_t HW = (size_t)pr.H * pr.W;
    const bool bt = transposes_in_flight(pass, pr);
    if (pass == 0) return bt ? 0 : round256((size_t)pr.N * HW * pr.C * 2);
    if (pass == 1) return (bt ? 0 : round256((size_t)pr.N * HW * pr.K * 2)) + round256((size_t)pr.K * pr.C * 2);
    const int s = wgrad_splits(pr);
    return s > 1 ? (size_t)s * pr.K * pr.C * sizeof(float) : 0;
}

hipError_t bf16_gemm_run(int pass, const Problem& pr, const void* in0, const void* in1, float* out, void* ws, hipStream_t st) {
    if (!bf16_gemm_accepts(pass, pr, in0, in1)) return hipErrorNotSupported;
    const int HW = pr.H * pr.W;
    GemmArgs a{};
    bool bt = false;
    a.HW = HW;
    a.out = out;
    hipError_t e = hipSuccess;
    if (pass < 2) {
        const int Cs = pass == 0 ? pr.C : pr.K, F = pass == 0 ? pr.K : pr.C;   // reduction / destination channels
        bt = transposes_in_flight(pass, pr);
        const uint16_t* bmat = static_cast<const uint16_t*>(in0);   // transposed in flight: the NCHW tensor itself
        size_t used = 0;
        if (!bt) {
            uint16_t* srcT = static_cast<uint16_t*>(ws);
            PackArgs pa{static_cast<const uint16_t*>(in0), srcT, pr.N, Cs, HW, (unsigned)((size_t)pr.N * Cs * HW * 2)};
            gemm_pack_nhwc_kernel<<<dim3((HW + 127) / 128, (Cs + 63) / 64, pr.N), 256, 0, st>>>(pa);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            bmat = srcT;
            used = round256((size_t)pr.N * HW * Cs * 2);
        }
        const uint16_t* wmat = static_cast<const uint16_t*>(in1);   // forward: w[K][C] as it is
        if (pass == 1) {
            uint16_t* wt = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(ws) + used);
            gemm_transpose_kernel<<<dim3((pr.C + 31) / 32, (pr.K + 31) / 32), 256, 0, st>>>(wmat, wt, pr.K, pr.C);
            if ((e = hipGetLastError()) != hipSuccess) return e;
            wmat = wt;
        }
        a.A = wmat; a.B = bmat;
        a.M = F; a.N = pr.N * HW; a.Kd = Cs;
        a.lda = Cs; a.ldb = Cs;
        a.batches = 1; a.splits = 1;
        a.mode = 0;
        a.out_bf16 = pr.out_bf16 ? 1 : 0;
        a.bias = pass == 0 ? pr.bias : nullptr;
        a.mask = pass == 1 ? static_cast<const uint16_t*>(pr.relu_mask) : nullptr;
    } else {
        a.A = static_cast<const uint16_t*>(in1);   // dy [N][K][HW]
        a.B = static_cast<const uint16_t*>(in0);   // x  [N][C][HW]
        a.M = pr.K; a.N = pr.C; a.Kd = HW;
        a.lda = HW; a.ldb = HW;
        a.a_batch = (long long)pr.K * HW; a.b_batch = (long long)pr.C * HW;
        a.batches = pr.N; a.splits = wgrad_splits(pr);
        a.mode = 1;
        if (a.splits > 1) a.out = ws;
    }
    a.tiles_m = (a.M + kEdge - 1) / kEdge;
    a.tiles_n = (a.N + kEdge - 1) / kEdge;
    const long long grid = (((long long)a.tiles_m * a.tiles_n * a.splits + 7) / 8) * 8;
    if (grid >= (1ll << 31)) return hipErrorNotSupported;
    if (bt) bf16_gemm_kernel<kEdge, kEdge, 4, 2, true><<<(unsigned)grid, NTHREADS, 0, st>>>(a);
    else bf16_gemm_kernel<kEdge, kEdge, 4, 2, false><<<(unsigned)grid, NTHREADS, 0, st>>>(a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (pass == 2 && a.splits > 1) {
        const size_t count = (size_t)pr.K * pr.C;
        gemm_reduce_splits_kernel<<<(unsigned)((count + 255) / 256), 256, 0, st>>>(static_cast<const float*>(ws), out, a.splits, count);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace miconv
