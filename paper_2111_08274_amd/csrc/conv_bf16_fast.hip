// bf16 kernels for the regular convolution layers of the bf16 configuration (3x3-style "same" convolutions, stride 1,
// channel counts that are multiples of 64): the bulk of the network's multiply-adds (paper Sec. 2.1: the forward and
// backward passes of every local step).
//
// The generic kernel spends ~20 vector-ALU instructions per MFMA on address arithmetic, conversions and a scalar
// epilogue, which caps the matrix cores near 10 %.  Here everything that does not change along K is computed once:
//   * weights are kept as two bf16 matrices per layer, refreshed from the fp32 master before every forward pass:
//       Wf[co][(tap, ci)]  for the forward pass and  Wb[ci][(flipped tap, co)]  for the data gradient, both
//       K-contiguous, so forward and data gradient are the SAME kernel (a stride-1 data gradient is a convolution
//       of dY with the flipped, transposed filter) and no conversion or transposition happens in the K loop;
//   * a thread's pixel offset and its 9-bit tap-validity mask are fixed; per slab only a wave-uniform tap delta is
//     added; all offsets are 32-bit;
//   * the MFMA operands are swapped (C^T = B^T A^T), which leaves 4 consecutive output channels in each lane, so
//     the epilogue stores 8 bytes (bf16) or 16 bytes (fp32) per lane instead of single elements.
// Kernels: conv_kernel (forward / data gradient, any image size), conv_patch_kernel (the same on 16- and 32-pixel-wide
// images with at most 128 channels: tile and border resident in LDS), wgrad_kernel (weight gradient: operands stored
// as they arrive and transposed by the LDS read), wgrad_taps_kernel (weight gradient on wide images: all taps from one
// patch), weight_prep_kernel.  Each has its own comment.
#include "train_kernels.h"
#include "conv_stats.h"

namespace hadfl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

constexpr int kBigLds = 2 * (256 + 256) * 72 * 2;   // dynamic LDS of the 256 x 256 kernel: two buffers of both operands
constexpr int kBigWgradLds = 2 * 64 * 2 * (256 + 32) * 2;   // 256 x 256 weight-gradient kernel: two buffers of 64 rows per operand

// Workgroups are handed to the eight accelerator dies in turn (workgroup i runs on die i % 8), and each die has its own
// L2.  The kernels below take a one-dimensional grid of 8 * chunk workgroups and give die d the logical work items
// [d * chunk, (d + 1) * chunk): consecutive items -- the tiles of one replica, which share its weights and activations --
// meet in one L2 instead of being fetched from memory by all eight.
constexpr int kDies = 8;
__device__ __forceinline__ unsigned logical_block()
{
    const unsigned chunk = gridDim.x / kDies;
    return (blockIdx.x % kDies) * chunk + blockIdx.x / kDies;
}
inline unsigned die_grid(long long items) { return (unsigned)((items + kDies - 1) / kDies * kDies); }

__device__ __forceinline__ u4 ldg16(const char* base, unsigned off) { return *reinterpret_cast<const u4*>(base + off); }

// ---------------------------------------------------------------------------------------------------------------
// Forward / data-gradient: out[m][n] = sum_k act[pixel(m) + tap(k)][c(k)] * wmat[n][k]
// ---------------------------------------------------------------------------------------------------------------
// Row order.  With a position table (p.perm) GEMM row m' = ps * B + b is image b at pixel position perm[ps], the
// positions sorted by their set of in-bounds taps.  A tile then holds one or two positions of many images instead of
// whole images, and the taps that are out of bounds for every row of the tile -- 5 of 9 in a corner -- are left out of
// the K loop: their products are exact zeros.  Without a table rows are pixels in memory order and all taps are visited.
struct RowGeo { int pix; unsigned tapmask; };
__device__ __forceinline__ RowGeo row_geo(const FastConvParams& p, int m)
{
    RowGeo g; g.pix = 0; g.tapmask = 0;
    if (m >= p.M) return g;
    const int hw = p.H * p.W;
    int pos;
    if (p.perm) { const int ps = m / p.B, b = m - ps * p.B; pos = p.perm[ps]; g.pix = b * hw + pos; }
    else { const int b = m / hw; pos = m - b * hw; g.pix = m; }
    const int y = pos / p.W, x = pos - y * p.W;
    for (int t = 0; t < p.R * p.S; ++t) {
        const int r = t / p.S, s = t - r * p.S;
        const int yy = y + r - p.pad, xx = x + s - p.pad;
        if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W) g.tapmask |= 1u << t;
    }
    return g;
}

// Taps some row of the tile [m0, m0 + rows) can reach
__device__ __forceinline__ unsigned tile_taps(const FastConvParams& p, int m0, int rows)
{
    const unsigned all = (p.R * p.S >= 32) ? 0xffffffffu : ((1u << (p.R * p.S)) - 1u);
    if (!p.perm) return all;
    const int last = min(m0 + rows, p.M) - 1;
    unsigned u = 0;
    for (int ps = m0 / p.B; ps <= last / p.B; ++ps) u |= p.posmask[ps];
    return u & all;
}

using conv_stats::store_column_stats;
using conv_stats::kStatLdsBytes;


// Tile BMT x BN, slabs of 64 along K, WGM x WGN waves (wave tile BMT/WGM x BN/WGN).  Eight neighbouring lanes read the
// full 128-byte line a row contributes to a slab.  NBUF = 1: one LDS buffer, the next slab waits in registers while the
// current one is multiplied, two barriers per slab.  NBUF = 2: the next slab is written to the other buffer before the
// current one is multiplied, one barrier per slab.  LDS rows are padded to 72 elements (conflict-free 16-byte reads).
// EPI 0: + bias, optional ReLU, store bf16;  EPI 1: optional mask, optional accumulate.
template <int BMT, int BN, int WGM, int WGN, int NBUF, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64, NBUF == 2 && WGM * WGN == 8 ? 1 : 2) void conv_kernel(FastConvParams p)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int BK2 = 64, LDQ = 72;
    constexpr int TM = BMT / WGM / 32, TN = BN / WGN / 32;
    constexpr int NQA = BMT * 8 / NT, NQB = BN * 8 / NT;      // 16-byte slots per thread: rows x 8 groups of 8 k
    static_assert(NQA >= 1 && NQB >= 1 && TM >= 1 && TN >= 1, "tile too small for the thread count");
    constexpr unsigned A_BUF = BMT * LDQ * 2, B_BUF = BN * LDQ * 2;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sAc = smem;                           // [NBUF][BMT][LDQ]
    char* const sBc = smem + NBUF * A_BUF;            // [NBUF][BN][LDQ]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    // logical item = (slot, column tile, row tile), row tiles fastest
    const unsigned tiles_m = (unsigned)(p.M + BMT - 1) / BMT, tiles_n = (unsigned)p.N / BN;
    const unsigned item = logical_block();
    if (item >= tiles_m * tiles_n * (unsigned)p.n_active) return;
    const int rep = p.order[item / (tiles_m * tiles_n)];
    const int m0 = (int)(item % tiles_m) * BMT, n0 = (int)((item / tiles_m) % tiles_n) * BN;
    const char* abase = (const char*)p.a + (long long)rep * p.a_rep * 4;
    const char* wbase = (const char*)(p.wmat + (long long)rep * p.wmat_rep);

    unsigned aoff[NQA], boff[NQB], sa_st[NQA], sb_st[NQB], tapmask[NQA];
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
        const int i = tid + q * NT;
        const int arow = i >> 3, kq = i & 7;
        const RowGeo g = row_geo(p, m0 + arow);
        tapmask[q] = g.tapmask;
        aoff[q] = (unsigned)(g.pix * p.C + kq * 8) * 2u;
        sa_st[q] = (unsigned)(arow * LDQ + kq * 8) * 2u;
    }
#pragma unroll
    for (int q = 0; q < NQB; ++q) {
        const int i = tid + q * NT;
        boff[q] = (unsigned)((n0 + (i >> 3)) * p.K + (i & 7) * 8) * 2u;
        sb_st[q] = (unsigned)((i >> 3) * LDQ + (i & 7) * 8) * 2u;
    }
    const unsigned a_rd = (unsigned)((wm * (BMT / WGM) + (lane & 31)) * LDQ + (lane >> 5) * 8) * 2u;
    const unsigned b_rd = (unsigned)((wn * (BN / WGN) + (lane & 31)) * LDQ + (lane >> 5) * 8) * 2u;

    // slabs: (tap, 64 channels) for the taps of this tile, taps ascending
    const unsigned taps = tile_taps(p, m0, BMT);
    const int nslab = __builtin_popcount(taps) * (p.C / BK2);
    unsigned taps_left = taps;
    int tap = taps ? __builtin_ctz(taps) : 0, c0 = 0;
    u4 ra[NQA], rb[NQB];
    auto load_tiles = [&]() {
        const int r = tap / p.S, s = tap - r * p.S;
        const int delta = (((r - p.pad) * p.W + (s - p.pad)) * p.C + c0) * 2;       // bytes, may be negative
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            u4 v = {0u, 0u, 0u, 0u};
            if ((tapmask[q] >> tap) & 1u) v = ldg16(abase, aoff[q] + (unsigned)delta);
            ra[q] = v;
        }
        const unsigned kb = (unsigned)(tap * p.C + c0) * 2u;
#pragma unroll
        for (int q = 0; q < NQB; ++q) rb[q] = ldg16(wbase, boff[q] + kb);
        c0 += BK2;
        if (c0 == p.C) {
            c0 = 0;
            taps_left &= taps_left - 1u;                 // drop the tap just finished
            tap = taps_left ? __builtin_ctz(taps_left) : 0;
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) *reinterpret_cast<u4*>(sAc + buf * A_BUF + sa_st[q]) = ra[q];
#pragma unroll
        for (int q = 0; q < NQB; ++q) *reinterpret_cast<u4*>(sBc + buf * B_BUF + sb_st[q]) = rb[q];
    };

    f16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto compute = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(sAc + buf * A_BUF + a_rd + (i * 32 * LDQ + ks * 16) * 2);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(sBc + buf * B_BUF + b_rd + (j * 32 * LDQ + ks * 16) * 2);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)      // operands swapped: the accumulator holds the transposed tile
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
    };

    if (nslab > 0) {
        load_tiles();
        if (NBUF == 1) {
            for (int t = 0; t < nslab; ++t) {
                __syncthreads();                               // every wave is done reading the previous slab
                store_tiles(0);
                __syncthreads();
                if (t + 1 < nslab) load_tiles();
                compute(0);
            }
        } else {
            store_tiles(0);
            if (nslab > 1) load_tiles();
            __syncthreads();
            for (int t = 0; t < nslab; ++t) {
                const int buf = t & 1;
                if (t + 1 < nslab) {
                    store_tiles(buf ^ 1);                      // slab t+1 (in registers since the previous iteration)
                    if (t + 2 < nslab) load_tiles();           // slab t+2 travels while slab t is multiplied
                }
                compute(buf);
                __syncthreads();
            }
        }
    }

    // ---- epilogue: lane holds output row (lane & 31) and channels 8*g + 4*(lane >> 5) + {0..3}, g = 0..3 ----
    char* obase = (char*)p.out + (long long)rep * p.out_rep * 4;
    const float* bias = (EPI == 0 && p.bias) ? p.bias + (long long)rep * p.bias_rep : nullptr;
    const char* mask = (EPI == 1 && p.mask) ? (const char*)p.mask + (long long)rep * p.mask_rep * 4 : nullptr;
    const bool stats = p.stat != nullptr;
    // data gradient with statistics: values of the tensor whose gradient this is (see FastConvParams::stat_y)
    const char* ysrc = (EPI == 1 && stats) ? (const char*)p.stat_y + (long long)rep * p.stat_y_rep * 4 : nullptr;
    const bool y_is_mask = mask != nullptr && ysrc == mask;
    float ss[TN][16], qq[TN][16];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int k = 0; k < 16; ++k) { ss[j][k] = 0.f; qq[j][k] = 0.f; }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mm = m0 + wm * (BMT / WGM) + i * 32 + (lane & 31);
        if (mm >= p.M) continue;
        int pix = mm;
        if (p.perm) { const int ps = mm / p.B, b = mm - ps * p.B; pix = b * p.H * p.W + p.perm[ps]; }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * (BN / WGN) + j * 32 + 8 * g + 4 * (lane >> 5);
                const unsigned o = (unsigned)(pix * p.N + n) * 2u;
                f4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                bf16x4 mk = {};
                f4 sh = {0.f, 0.f, 0.f, 0.f};                  // what the statistics are centred on: the bias
                if (EPI == 0) {
                    if (bias) { sh = *reinterpret_cast<const f4*>(bias + n); v += sh; }
                    if (p.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                } else {
                    if (mask) {
                        mk = *reinterpret_cast<const bf16x4*>(mask + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (!((float)mk[e] > 0.f)) v[e] = 0.f;
                    }
                    if (p.accumulate) {
                        const bf16x4 old = *reinterpret_cast<const bf16x4*>(obase + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (float)old[e];
                    }
                }
                bf16x4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (__bf16)v[e];
                *reinterpret_cast<bf16x4*>(obase + o) = r;
                if (stats) {
                    if (EPI == 0) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { const float f = (float)r[e] - sh[e]; ss[j][4 * g + e] += f; qq[j][4 * g + e] += f * f; }
                    } else {
                        // the mask of a fused ReLU is that very tensor: its values are already here
                        const bf16x4 yv = y_is_mask ? mk : *reinterpret_cast<const bf16x4*>(ysrc + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float yy = (float)yv[e];
                            const float f = (p.stat_relu && !(yy > 0.f)) ? 0.f : (float)r[e];
                            ss[j][4 * g + e] += f; qq[j][4 * g + e] += f * yy;
                        }
                    }
                }
            }
        }
    }
    if (stats) {
        // (the launcher asks for the larger of the K loop's LDS and kStatLdsBytes)
        __syncthreads();                                      // every wave is past its last operand read
        const int slot = (int)(item / (tiles_m * tiles_n));
        store_column_stats<TN, WGM, WGN>(ss, qq, reinterpret_cast<float*>(smem), wave, lane, p.stat + (long long)slot * p.stat_rep,
                                         m0 / BMT, n0 + wn * (BN / WGN), p.N);
    }
}

// Wide images (16 or 32 pixels per row) with few channels move more bytes per multiply-add than the general kernel can
// fetch: it reads every activation once per tap.  Here a workgroup owns BMT consecutive pixels of one image (whole
// rows), loads them ONCE per 64-channel slice together with their one-pixel border (zeros outside the image) into
// LDS, and serves all R*S taps from that patch by shifting the row it reads; only the weights still stream per tap.
// IW = image width; 3x3-style filters with pad = (R-1)/2 <= 1.
// With 16-pixel rows the 32 lanes of an operand read span two patch rows; the read only runs at full rate when the
// second row starts a multiple of 256 bytes after the first (measured: half rate otherwise), so patch rows are padded
// to kPatchRowBytes<16>.
template <int IW> constexpr int kPatchRowBytes = IW == 16 ? ((IW + 2) * 144 + 255) / 256 * 256 : (IW + 2) * 144;
// TPS = taps per step (R * S a multiple of it): the weights of TPS taps of a channel slice are staged together, so a
// wave multiplies TPS * 64 contraction indices between two barriers instead of 64.
template <int IW, int BN, int WGM, int EPI, int TPS = 1, int BMT = 256>
__global__ __launch_bounds__(256, BMT == 256 ? 2 : 4) void conv_patch_kernel(FastConvParams p)
{
    constexpr int LDQ = 72, PW = IW + 2, TR = BMT / IW, PR = (TR + 2) * PW;   // patch: (TR + 2) x (IW + 2) pixels
    constexpr int RPB = kPatchRowBytes<IW>;                   // bytes per patch row
    constexpr int WGN = 4 / WGM;                              // wave grid WGM x WGN, wave tile (BMT / WGM) x (BN / WGN)
    constexpr int TM = BMT / WGM / 32, TN = BN / WGN / 32;
    static_assert(TM >= 1 && TN >= 1, "");
    constexpr int NQB = BN * 8 / 256;
    constexpr int NQP = (PR * 8 + 255) / 256;                 // patch slots per thread
    constexpr unsigned P_BYTES = (TR + 2) * RPB;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sP = smem;                                    // [TR + 2][RPB]: rows of PW pixels x LDQ, activations with border
    char* const sB = smem + P_BYTES;                          // [TPS][BN][LDQ] weights of TPS taps of one channel slice
    constexpr unsigned B_TAP = BN * LDQ * 2;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    const unsigned tiles_m = (unsigned)p.M / BMT, tiles_n = (unsigned)p.N / BN;
    const unsigned item = logical_block();
    if (item >= tiles_m * tiles_n * (unsigned)p.n_active) return;
    const int rep = p.order[item / (tiles_m * tiles_n)];
    const int m0 = (int)(item % tiles_m) * BMT, n0 = (int)((item / tiles_m) % tiles_n) * BN;
    const int img = m0 / (p.H * IW), y0 = (m0 - img * p.H * IW) / IW;          // first image row of the tile
    const char* abase = (const char*)p.a + (long long)rep * p.a_rep * 4;
    const char* wbase = (const char*)(p.wmat + (long long)rep * p.wmat_rep);

    // patch slots: slot i = (patch pixel i / 8, 16-byte channel group i % 8)
    int poff[NQP];                                            // byte offset of the source pixel's slice start, or -1
    unsigned pst[NQP];
#pragma unroll
    for (int q = 0; q < NQP; ++q) {
        const int i = tid + q * 256, pr = i >> 3, kq = i & 7;
        const int py = pr / PW, px = pr - py * PW;
        const int yy = y0 - 1 + py, xx = px - 1;
        const bool ok = pr < PR && yy >= 0 && yy < p.H && xx >= 0 && xx < IW;
        poff[q] = ok ? (((img * p.H + yy) * IW + xx) * p.C + kq * 8) * 2 : -1;
        pst[q] = (unsigned)(py * RPB + (px * LDQ + kq * 8) * 2);
    }
    unsigned boff[NQB], sb_st[NQB];
#pragma unroll
    for (int q = 0; q < NQB; ++q) {
        const int i = tid + q * 256;
        boff[q] = (unsigned)((n0 + (i >> 3)) * p.K + (i & 7) * 8) * 2u;
        sb_st[q] = (unsigned)((i >> 3) * LDQ + (i & 7) * 8) * 2u;
    }
    unsigned a_rd[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int pm = wm * (BMT / WGM) + i * 32 + (lane & 31);
        a_rd[i] = (unsigned)((pm / IW) * RPB + ((pm % IW) * LDQ + (lane >> 5) * 8) * 2);
    }
    const unsigned b_rd = (unsigned)((wn * (BN / WGN) + (lane & 31)) * LDQ + (lane >> 5) * 8) * 2u;

    f16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int taps = p.R * p.S;
    const int off0 = 1 - p.pad;                               // patch border is one pixel: tap (r, s) reads patch pixel + (r + off0, s + off0)
    // One step = TPS taps of one 64-channel slice: TPS * 64 contraction indices, too little matrix work to cover the
    // latency of its own weight load.  The weights of step i are therefore requested D steps ahead, into a ring of
    // register sets.
    constexpr int D = TPS > 1 ? 2 : (BN <= 64 ? 4 : 2);
    const int spt = taps / TPS;                               // steps per channel slice
    const int steps = (p.C / 64) * spt;
    u4 rb[D][TPS][NQB];
    auto load_w = [&](int step, u4 (&dst)[TPS][NQB]) {
        const int sl = step / spt, tap0 = (step - sl * spt) * TPS;
#pragma unroll
        for (int t = 0; t < TPS; ++t) {
            const unsigned kb = (unsigned)((tap0 + t) * p.C + sl * 64) * 2u;
#pragma unroll
            for (int q = 0; q < NQB; ++q) dst[t][q] = ldg16(wbase, boff[q] + kb);
        }
    };
#pragma unroll
    for (int d = 0; d < D; ++d)
        if (d < steps) load_w(d, rb[d]);
    for (int step0 = 0; step0 < steps; step0 += D) {
#pragma unroll
        for (int d = 0; d < D; ++d) {
            const int step = step0 + d;
            if (step >= steps) break;
            const int sl = step / spt, tap0 = (step - sl * spt) * TPS;
            if (tap0 == 0) {
                u4 rp[NQP];
#pragma unroll
                for (int q = 0; q < NQP; ++q) {
                    u4 v = {0u, 0u, 0u, 0u};
                    if (poff[q] >= 0) v = ldg16(abase, (unsigned)(poff[q] + sl * 128));
                    rp[q] = v;
                }
                __syncthreads();                              // every wave is done with the previous slice
#pragma unroll
                for (int q = 0; q < NQP; ++q)
                    if (tid + q * 256 < PR * 8) *reinterpret_cast<u4*>(sP + pst[q]) = rp[q];
            } else {
                __syncthreads();                              // every wave is done reading the previous step's weights
            }
#pragma unroll
            for (int t = 0; t < TPS; ++t)
#pragma unroll
                for (int q = 0; q < NQB; ++q) *reinterpret_cast<u4*>(sB + t * B_TAP + sb_st[q]) = rb[d][t][q];
            __syncthreads();
            if (step + D < steps) load_w(step + D, rb[d]);
#pragma unroll
            for (int t = 0; t < TPS; ++t) {
                const int tap = tap0 + t;
                const int r = tap / p.S, s2 = tap - r * p.S;
                const unsigned toff = (unsigned)((r + off0) * RPB + (s2 + off0) * LDQ * 2);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    bf16x8 a[TM], b[TN];
#pragma unroll
                    for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(sP + a_rd[i] + toff + ks * 32);
#pragma unroll
                    for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(sB + t * B_TAP + b_rd + (j * 32 * LDQ + ks * 16) * 2);
#pragma unroll
                    for (int i = 0; i < TM; ++i)
#pragma unroll
                        for (int j = 0; j < TN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: lane holds output row (lane & 31) and channels 8*g + 4*(lane >> 5) + {0..3}, g = 0..3 ----
    char* obase = (char*)p.out + (long long)rep * p.out_rep * 4;
    const float* bias = (EPI == 0 && p.bias) ? p.bias + (long long)rep * p.bias_rep : nullptr;
    const char* mask = (EPI == 1 && p.mask) ? (const char*)p.mask + (long long)rep * p.mask_rep * 4 : nullptr;
    const bool stats = p.stat != nullptr;
    // data gradient with statistics: values of the tensor whose gradient this is (see FastConvParams::stat_y)
    const char* ysrc = (EPI == 1 && stats) ? (const char*)p.stat_y + (long long)rep * p.stat_y_rep * 4 : nullptr;
    const bool y_is_mask = mask != nullptr && ysrc == mask;
    float ss[TN][16], qq[TN][16];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) { ss[j][kk] = 0.f; qq[j][kk] = 0.f; }
#pragma unroll
    for (int i = 0; i < TM; ++i) {
        const int mm = m0 + wm * (BMT / WGM) + i * 32 + (lane & 31);
#pragma unroll
        for (int j = 0; j < TN; ++j) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn * (BN / WGN) + j * 32 + 8 * g + 4 * (lane >> 5);
                const unsigned o = (unsigned)(mm * p.N + n) * 2u;
                f4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                bf16x4 mk = {};
                f4 sh = {0.f, 0.f, 0.f, 0.f};                  // what the statistics are centred on: the bias
                if (EPI == 0) {
                    if (bias) { sh = *reinterpret_cast<const f4*>(bias + n); v += sh; }
                    if (p.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                } else {
                    if (mask) {
                        mk = *reinterpret_cast<const bf16x4*>(mask + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (!((float)mk[e] > 0.f)) v[e] = 0.f;
                    }
                    if (p.accumulate) {
                        const bf16x4 old = *reinterpret_cast<const bf16x4*>(obase + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) v[e] += (float)old[e];
                    }
                }
                bf16x4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (__bf16)v[e];
                *reinterpret_cast<bf16x4*>(obase + o) = r;
                if (stats) {
                    if (EPI == 0) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) { const float f = (float)r[e] - sh[e]; ss[j][4 * g + e] += f; qq[j][4 * g + e] += f * f; }
                    } else {
                        // the mask of a fused ReLU is that very tensor: its values are already here
                        const bf16x4 yv = y_is_mask ? mk : *reinterpret_cast<const bf16x4*>(ysrc + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float yy = (float)yv[e];
                            const float f = (p.stat_relu && !(yy > 0.f)) ? 0.f : (float)r[e];
                            ss[j][4 * g + e] += f; qq[j][4 * g + e] += f * yy;
                        }
                    }
                }
            }
        }
    }
    if (stats) {
        // (the launcher asks for the larger of the K loop's LDS and kStatLdsBytes)
        __syncthreads();                                      // every wave is past its last operand read
        const int slot = (int)(item / (tiles_m * tiles_n));
        store_column_stats<TN, WGM, WGN>(ss, qq, reinterpret_cast<float*>(smem), wave, lane, p.stat + (long long)slot * p.stat_rep,
                                         m0 / BMT, n0 + wn * (BN / WGN), p.N);
    }
}

// ---------------------------------------------------------------------------------------------------------------
// Weight gradient: dW[m = (tap, ci) | bias row][n = co] = sum over pixels k of x[k + tap][ci] * dy[k][co]
// ---------------------------------------------------------------------------------------------------------------
// Both operands are contiguous along their row index (channels) and the contraction runs over pixels, so the tiles
// are stored in LDS as they arrive, [k][row] with 16-byte stores, and transposed on the way OUT of LDS with
// ds_read_b64_tr_b16: within a group of 16 lanes, lane i receives element (i % 4) of the 8 bytes addressed by lane
// 4*j + i/4, for j = 0..3.  Pointing lane L at row k0 + L/4, columns 4*(L%4).. of a 16-column block therefore hands
// lane i the four consecutive k of column i -- half of an MFMA operand.
typedef short s4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v lds_s4v;

__device__ __forceinline__ bf16x8 lds_read_tr8(const char* base, unsigned off, unsigned row_pitch_bytes)
{
    // base + off addresses this lane's 8 bytes in row k0; rows k0+4.. supply the upper four k
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v*)(base + off));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v*)(base + off + 4 * row_pitch_bytes));
    typedef short s8v __attribute__((ext_vector_type(8)));
    const s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

// Epilogue of the weight-gradient kernels.  A lane holds row (lane & 31) of a 32 x 32 block and 16 of its columns in
// groups of four; stored like that, one instruction would touch 32 rows with 32 bytes each.  Each wave passes its blocks
// through a private piece of LDS (free once every wave is past the last barrier of the K loop) and takes them back with
// eight lanes per row, so that global accesses cover whole 128-byte lines.  Rows from m_end on are not stored.
// With sgd_w set the block is a complete gradient and the update (buf = momentum*buf + g; w -= lr*buf) is applied instead.
constexpr int kStagePitch = 36;                              // floats per staged row (144 bytes: conflict-free 16-byte writes)
__device__ __forceinline__ void store_block32(const f16& acc, float* stage, int lane, int m_base, int m_end, int n_base,
                                              const FastWgradParams& p, float* obase, float* sgd_w, float* sgd_buf)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        *reinterpret_cast<f4*>(stage + (lane & 31) * kStagePitch + 8 * q + 4 * (lane >> 5)) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int rr = (lane >> 3) + 8 * t, cc = (lane & 7) * 4;
        const f4 v = *reinterpret_cast<const f4*>(stage + rr * kStagePitch + cc);
        const int mm = m_base + rr;
        if (mm >= m_end) continue;
        const long long o = (long long)mm * p.N + n_base + cc;
        if (sgd_w) {
            f4 d = v;
            if (sgd_buf) { d = *reinterpret_cast<const f4*>(sgd_buf + o) * p.momentum + d; *reinterpret_cast<f4*>(sgd_buf + o) = d; }
            *reinterpret_cast<f4*>(sgd_w + o) = *reinterpret_cast<const f4*>(sgd_w + o) - d * p.lr;
        } else {
            *reinterpret_cast<f4*>(obase + o) = v;
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The fused update of one 32 x 32 block in two steps, so that the parameter and momentum loads of the NEXT block are in
// flight while the current one is staged, updated and stored: a wave that loads, computes and stores block after block
// keeps only 2 KiB in flight and the epilogue of the short-contraction layers runs at a fraction of the memory rate.
struct UpdateOperands { f4 w[4], b[4]; };
__device__ __forceinline__ void fetch_update_operands(UpdateOperands& u, int lane, int m_base, int m_end, int n_base, int N,
                                                      const float* sgd_w, const float* sgd_buf)
{
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int mm = m_base + (lane >> 3) + 8 * t;
        const long long o = (long long)mm * N + n_base + (lane & 7) * 4;
        u.w[t] = f4{0.f, 0.f, 0.f, 0.f}; u.b[t] = f4{0.f, 0.f, 0.f, 0.f};
        if (mm < m_end) {
            u.w[t] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(sgd_w + o));          // streamed once per step
            if (sgd_buf) u.b[t] = __builtin_nontemporal_load(reinterpret_cast<const f4*>(sgd_buf + o));
        }
    }
}
__device__ __forceinline__ void update_block32(const f16& acc, const UpdateOperands& u, float* stage, int lane, int m_base, int m_end,
                                               int n_base, const FastWgradParams& p, float* sgd_w, float* sgd_buf)
{
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const f4 v = {acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        *reinterpret_cast<f4*>(stage + (lane & 31) * kStagePitch + 8 * q + 4 * (lane >> 5)) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        const int rr = (lane >> 3) + 8 * t, cc = (lane & 7) * 4;
        f4 d = *reinterpret_cast<const f4*>(stage + rr * kStagePitch + cc);
        const int mm = m_base + rr;
        if (mm >= m_end) continue;
        const long long o = (long long)mm * p.N + n_base + cc;
        if (sgd_buf) { d = u.b[t] * p.momentum + d; __builtin_nontemporal_store(d, reinterpret_cast<f4*>(sgd_buf + o)); }
        __builtin_nontemporal_store(u.w[t] - d * p.lr, reinterpret_cast<f4*>(sgd_w + o));
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Tile BMT x BN, WGM x WGN waves, slabs of BKT contraction indices, two LDS buffers.
template <int BMT, int BN, int WGM, int WGN, int BKT>
__global__ __launch_bounds__(WGM * WGN * 64, WGM * WGN == 8 ? 1 : 3) void wgrad_kernel(FastWgradParams p)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int TM = BMT / WGM / 32, TN = BN / WGN / 32;
    // row pitches in bytes, 64 modulo 256: the 4 rows x 64 bytes that 32 lanes of a transposing read touch land in
    // distinct banks
    constexpr int PA = (BMT + 32) * 2, PB = (BN + 32) * 2;
    constexpr int AOCT = BMT / 8, BOCT = BN / 8;            // 16-byte octets per contraction row
    constexpr int AROWS = NT / AOCT, BROWS = NT / BOCT;     // contraction rows the threads cover per pass
    constexpr int NQA = BKT / AROWS, NQB = BKT / BROWS;     // passes (slots per thread)
    static_assert(NT % AOCT == 0 && NT % BOCT == 0 && NQA >= 1 && NQB >= 1 && BKT % AROWS == 0 && BKT % BROWS == 0, "");
    constexpr unsigned A_BUF = BKT * PA, B_BUF = BKT * PB;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sA = smem;                                  // [2][BKT][PA]
    char* const sB = smem + 2 * A_BUF;                      // [2][BKT][PB]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    // logical item = (slot, split, tile): the tiles of one split of one replica read the same pixels
    const unsigned tiles_n = (unsigned)p.N / BN, tiles = (unsigned)((p.M + BMT - 1) / BMT) * tiles_n;
    const unsigned item = logical_block();
    if (item >= tiles * (unsigned)p.splits * (unsigned)p.n_active) return;
    const int g = (int)(item / (tiles * (unsigned)p.splits));
    const int rep = p.order[g];
    const unsigned tile = item % tiles;
    const int m0 = (int)(tile / tiles_n) * BMT, n0 = (int)(tile % tiles_n) * BN;
    const int split = (int)((item / tiles) % (unsigned)p.splits);
    const int kbeg = split * p.kchunk, kend = min(p.K, kbeg + p.kchunk);
    const char* xbase = (const char*)p.x + (long long)rep * p.x_rep * 4;
    const char* dbase = (const char*)p.dy + (long long)rep * p.dy_rep * 4;

    // A slots of this thread: octet of rows (tid % AOCT) at contraction rows tid / AOCT + AROWS * q
    const int oct = tid % AOCT, krow = tid / AOCT;
    const int am = m0 + oct * 8;
    const int mw = p.R * p.S * p.C;
    const int atap = am / p.C, aci = am - atap * p.C;
    const int ar = atap / p.S, as = atap - ar * p.S;
    const int ady = ar - p.pad, adx = as - p.pad;
    const int a_kind = am < mw ? 0 : (am == mw && p.has_bias ? 1 : 2);      // 0 data, 1 bias row of ones, 2 nothing
    const int a_shift = ((ady * p.W + adx) * p.C + aci) * 2;
    const unsigned sa_st = (unsigned)(krow * PA + oct * 16);
    // B slots: octet tid % BOCT at contraction rows tid / BOCT + BROWS * q
    const int boct = tid % BOCT, bkrow = tid / BOCT;
    const unsigned sb_st = (unsigned)(bkrow * PB + boct * 16);
    const unsigned bnoff = (unsigned)(n0 + boct * 8) * 2u;
    // operand read offsets (see lds_read_tr8): lane L of a 16-lane group points at row L/4, columns 4*(L%4)
    const unsigned rd_lane = (unsigned)(((lane >> 5) * 8 + ((lane & 15) >> 2)));
    const unsigned a_rd = rd_lane * PA + (unsigned)(wm * (BMT / WGM) + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2u;
    const unsigned b_rd = rd_lane * PB + (unsigned)(wn * (BN / WGN) + ((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2u;

    // Contraction order.  With a position table, index k' = ps * B + b is image b at pixel perm[ps] (B a multiple of
    // the slab length, so a slab holds one position); a slab whose position cannot reach any tap of this row tile
    // contributes exact zeros and is left out.  Without a table k' is the pixel index and every slab is visited.
    const int hw = p.H * p.W;
    unsigned tile_tapbits = 0xffffffffu;
    if (p.perm && !(p.has_bias && m0 <= mw && mw < m0 + BMT)) {
        const int tlo = m0 / p.C, thi = min(m0 + BMT - 1, mw - 1) / p.C;
        tile_tapbits = (thi >= 31 ? 0xffffffffu : ((2u << thi) - 1u)) & ~((1u << tlo) - 1u);
    }
    auto next_slab = [&](int k) {
        if (p.perm)
            while (k < kend && !(p.posmask[k / p.B] & tile_tapbits)) k += BKT;
        return k;
    };
    u4 ra[NQA], rb[NQB];
    auto load_tiles = [&](int k0) {
        int bbase = 0, pos = 0;
        if (p.perm) { const int ps = k0 / p.B; bbase = k0 - ps * p.B; pos = p.perm[ps]; }
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int kr = krow + AROWS * q, kk = k0 + kr;
            u4 v = {0u, 0u, 0u, 0u};
            if (kk < kend) {
                if (a_kind == 0) {
                    int pix = kk, ppos = kk;
                    if (p.perm) { pix = (bbase + kr) * hw + pos; ppos = pos; }
                    const int yy = ((ppos >> p.w_shift) & (p.H - 1)) + ady, xx = (ppos & (p.W - 1)) + adx;
                    if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                        v = ldg16(xbase, (unsigned)(pix * p.C * 2 + a_shift));
                } else if (a_kind == 1) {
                    v[0] = 0x3f80u;                 // bf16 1.0 in the first of the 8 rows
                }
            }
            ra[q] = v;
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) {
            const int kr = bkrow + BROWS * q, kk = k0 + kr;
            u4 w = {0u, 0u, 0u, 0u};
            if (kk < kend) {
                int pix = kk;
                if (p.perm) pix = (bbase + kr) * hw + pos;
                w = ldg16(dbase, (unsigned)(pix * p.N) * 2u + bnoff);
            }
            rb[q] = w;
        }
    };
    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) *reinterpret_cast<u4*>(sA + buf * A_BUF + sa_st + AROWS * q * PA) = ra[q];
#pragma unroll
        for (int q = 0; q < NQB; ++q) *reinterpret_cast<u4*>(sB + buf * B_BUF + sb_st + BROWS * q * PB) = rb[q];
    };

    f16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    int k0 = next_slab(kbeg), buf = 0;
    if (k0 < kend) { load_tiles(k0); store_tiles(0); }
    __syncthreads();
    while (k0 < kend) {
        const int k1 = next_slab(k0 + BKT);
        if (k1 < kend) load_tiles(k1);
#pragma unroll
        for (int ks = 0; ks < BKT / 16; ++ks) {
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = lds_read_tr8(sA + buf * A_BUF, a_rd + ks * 16 * PA + i * 64, PA);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = lds_read_tr8(sB + buf * B_BUF, b_rd + ks * 16 * PB + j * 64, PB);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
        }
        if (k1 < kend) store_tiles(buf ^ 1);
        __syncthreads();
        buf ^= 1; k0 = k1;
    }

    // ---- epilogue (see store_block32) ----
    float* obase = (p.splits > 1) ? p.out + (long long)g * p.out_rep + (long long)split * p.out_split
                                  : p.out + (long long)rep * p.out_rep;
    float* const sgd_w = (p.splits == 1 && p.sgd_w) ? p.sgd_w + (long long)rep * p.out_rep : nullptr;
    float* const sgd_buf = (sgd_w && p.sgd_buf) ? p.sgd_buf + (long long)rep * p.out_rep : nullptr;
    static_assert((size_t)NT / 64 * 32 * kStagePitch * 4 <= 2 * (size_t)(A_BUF + B_BUF), "staging area does not fit the LDS of the K loop");
    float* const stage = reinterpret_cast<float*>(smem) + wave * (32 * kStagePitch);
    if (sgd_w) {
        const int mb = m0 + wm * (BMT / WGM), nb = n0 + wn * (BN / WGN);
        UpdateOperands u[2];
        fetch_update_operands(u[0], lane, mb, p.M, nb, p.N, sgd_w, sgd_buf);
#pragma unroll
        for (int k = 0; k < TM * TN; ++k) {
            if (k + 1 < TM * TN)
                fetch_update_operands(u[(k + 1) & 1], lane, mb + ((k + 1) / TN) * 32, p.M, nb + ((k + 1) % TN) * 32, p.N, sgd_w, sgd_buf);
            update_block32(acc[k / TN][k % TN], u[k & 1], stage, lane, mb + (k / TN) * 32, p.M, nb + (k % TN) * 32, p, sgd_w, sgd_buf);
        }
        return;
    }
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
            store_block32(acc[i][j], stage, lane, m0 + wm * (BMT / WGM) + i * 32, p.M, n0 + wn * (BN / WGN) + j * 32, p, obase, sgd_w, sgd_buf);
}

// Wide images (16 or 32 pixels per row) with few channels: the kernel above reads every activation once per tap and
// is bound by that traffic.  Here a workgroup owns ALL taps of a 64-channel input slice against 64 output channels:
// per slab of 32 pixels (whole image rows) it loads those rows with their one-pixel border ONCE into LDS and forms
// the nine shifted operands from that patch by offsetting the row the transposing read points at.
// Waves: (input-channel half, output-channel half); each keeps nine 32 x 32 blocks (one per tap), the waves of the
// first half of slice 0 also the bias row.  IW = image width (a slab is 32 / IW whole rows of one image, so the image
// height is a multiple of that); 3 x 3 filter, pad 1.
template <int IW>
__global__ __launch_bounds__(256, 2) void wgrad_taps_kernel(FastWgradParams p)
{
    constexpr int PW = IW + 2, SR = 32 / IW, PP = (SR + 2) * PW;      // patch: (SR + 2) x (IW + 2) pixels
    constexpr int PT = 192;                                         // bytes per patch pixel / dY row: 64 channels + pad (64 mod 256)
    constexpr int NQP = (PP * 8 + 255) / 256;
    constexpr unsigned P_BUF = PP * PT, D_BUF = 32 * PT;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sP = smem;                                          // [2][PP][PT]
    char* const sD = smem + 2 * P_BUF;                              // [2][32][PT]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ch = wave & 1, nh = wave >> 1;
    // logical item = (slot, split, input slice, output tile)
    const unsigned cslices = (unsigned)p.C / 64, ntiles = (unsigned)p.N / 64, tiles = cslices * ntiles;
    const unsigned item = logical_block();
    if (item >= tiles * (unsigned)p.splits * (unsigned)p.n_active) return;
    const int g = (int)(item / (tiles * (unsigned)p.splits));
    const int rep = p.order[g];
    const int split = (int)((item / tiles) % (unsigned)p.splits);
    const int ci0 = (int)((item % tiles) / ntiles) * 64, n0 = (int)(item % ntiles) * 64;
    const int kbeg = split * p.kchunk, kend = min(p.K, kbeg + p.kchunk);
    const char* xbase = (const char*)p.x + (long long)rep * p.x_rep * 4;
    const char* dbase = (const char*)p.dy + (long long)rep * p.dy_rep * 4;
    const int hw = p.H * IW;

    // patch slots: slot i = (patch pixel i / 8, 16-byte channel group i % 8)
    int prel[NQP], pyy[NQP];                                        // source offset relative to the slab, row offset (or a value that never fits)
    unsigned pst[NQP];
#pragma unroll
    for (int q = 0; q < NQP; ++q) {
        const int i = tid + q * 256, pp = i >> 3, kq = i & 7;
        const int py = pp / PW, px = pp - py * PW;
        const bool ok = pp < PP && px >= 1 && px <= IW;
        prel[q] = (((py - 1) * IW + (px - 1)) * p.C + ci0 + kq * 8) * 2;
        pyy[q] = ok ? py - 1 : -(1 << 20);
        pst[q] = (unsigned)(pp * PT + kq * 16);
    }
    const unsigned dst = (unsigned)((tid >> 3) * PT + (tid & 7) * 16);
    const unsigned doff = (unsigned)(((tid >> 3) * p.N + n0 + (tid & 7) * 8) * 2);

    u4 rp[NQP], rd;
    auto load_slab = [&](int k0) {
        const int b = k0 / hw, y0 = (k0 - b * hw) / IW;
        const int base = (b * hw + y0 * IW) * p.C * 2;
#pragma unroll
        for (int q = 0; q < NQP; ++q) {
            u4 v = {0u, 0u, 0u, 0u};
            const int yy = y0 + pyy[q];
            if (yy >= 0 && yy < p.H) v = ldg16(xbase, (unsigned)(base + prel[q]));
            rp[q] = v;
        }
        rd = ldg16(dbase, (unsigned)(k0 * p.N * 2) + doff);
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int q = 0; q < NQP; ++q)
            if (tid + q * 256 < PP * 8) *reinterpret_cast<u4*>(sP + buf * P_BUF + pst[q]) = rp[q];
        *reinterpret_cast<u4*>(sD + buf * D_BUF + dst) = rd;
    };

    // operand reads (see lds_read_tr8): the lane's contraction index inside a 16-block and its 4-column group
    const int kl = (lane >> 5) * 8 + ((lane & 15) >> 2);
    const unsigned col = (unsigned)((((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2);
    unsigned a_rd[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        const int k = ks * 16 + kl;
        a_rd[ks] = (unsigned)(((k / IW) * PW + (k % IW)) * PT) + (unsigned)(ch * 64) + col;
    }
    const unsigned b_rd = (unsigned)(kl * PT) + (unsigned)(nh * 64) + col;
    const bool with_bias = p.has_bias && ci0 == 0 && ch == 0;
    bf16x8 ones;
#pragma unroll
    for (int e = 0; e < 8; ++e) ones[e] = (__bf16)((lane & 31) == 0 ? 1.0f : 0.0f);

    f16 acc[9], accb;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[t][v] = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) accb[v] = 0.f;

    int buf = 0;
    if (kbeg < kend) { load_slab(kbeg); store_slab(0); }
    __syncthreads();
    for (int k0 = kbeg; k0 < kend; k0 += 32) {
        if (k0 + 32 < kend) load_slab(k0 + 32);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 b = lds_read_tr8(sD + buf * D_BUF, b_rd + ks * 16 * PT, PT);
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const bf16x8 a = lds_read_tr8(sP + buf * P_BUF, a_rd[ks] + (unsigned)(((t / 3) * PW + (t % 3)) * PT), PT);
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, a, acc[t], 0, 0, 0);
            }
            if (with_bias) accb = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, ones, accb, 0, 0, 0);
        }
        if (k0 + 32 < kend) store_slab(buf ^ 1);
        __syncthreads();
        buf ^= 1;
    }

    float* obase = (p.splits > 1) ? p.out + (long long)g * p.out_rep + (long long)split * p.out_split
                                  : p.out + (long long)rep * p.out_rep;
    float* const sgd_w = (p.splits == 1 && p.sgd_w) ? p.sgd_w + (long long)rep * p.out_rep : nullptr;
    float* const sgd_buf = (sgd_w && p.sgd_buf) ? p.sgd_buf + (long long)rep * p.out_rep : nullptr;
    static_assert(4 * 32 * kStagePitch * 4 <= 2 * (P_BUF + D_BUF), "staging area does not fit the LDS of the K loop");
    float* const stage = reinterpret_cast<float*>(smem) + wave * (32 * kStagePitch);
    const int mw = 9 * p.C;
#pragma unroll
    for (int t = 0; t < 9; ++t)
        store_block32(acc[t], stage, lane, t * p.C + ci0 + ch * 32, mw, n0 + nh * 32, p, obase, sgd_w, sgd_buf);
    if (with_bias) store_block32(accb, stage, lane, mw, mw + 1, n0 + nh * 32, p, obase, sgd_w, sgd_buf);
}

// ---------------------------------------------------------------------------------------------------------------
// Weight preparation: fp32 master W[tap][ci][co] -> Wf[co][tap*C + ci] and Wb[ci][(T-1-tap)*N + co], both bf16.
// A workgroup handles one tap and a 64 x 64 (ci, co) tile: 256-byte reads, whole 128-byte lines written to both copies.
// ---------------------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void weight_prep_kernel(WeightPrepParams p)
{
    __shared__ float tile[64][65];
    const int rep = p.order[blockIdx.z];
    const int taps = p.taps;
    const int tap = blockIdx.y % taps, cot = blockIdx.y / taps;
    const int ci0 = blockIdx.x * 64, co0 = cot * 64;
    const float* w = p.w + (long long)rep * p.w_rep + ((long long)tap * p.C) * p.N;
    __bf16* wf = p.wf + (long long)rep * p.wbf_rep;
    __bf16* wb = p.wb + (long long)rep * p.wbf_rep;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int K = taps * p.C, Kb = taps * p.N;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ci = ci0 + ty + 4 * r;
        const float v = __builtin_nontemporal_load(w + (long long)ci * p.N + co0 + tx);    // the master weights are read once
        tile[ty + 4 * r][tx] = v;
        wb[(long long)ci * Kb + (taps - 1 - tap) * p.N + co0 + tx] = (__bf16)v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int co = co0 + ty + 4 * r;
        wf[(long long)co * K + tap * p.C + ci0 + tx] = (__bf16)tile[tx][ty + 4 * r];
    }
}

template <int BMT, int BN, int WGM, int WGN, int NBUF>
void launch_conv_t(const FastConvParams& p, int epi, int n_active, hipStream_t s)
{
    constexpr size_t loop_lds = (size_t)NBUF * (BMT + BN) * 72 * 2, stat_lds = kStatLdsBytes<BN / WGN / 32, WGM, WGN>;
    constexpr size_t lds = loop_lds > stat_lds ? loop_lds : stat_lds;
    const dim3 grid(die_grid((long long)((p.M + BMT - 1) / BMT) * (p.N / BN) * n_active)), block(WGM * WGN * 64);
    if (epi == 0) hipLaunchKernelGGL((conv_kernel<BMT, BN, WGM, WGN, NBUF, 0>), grid, block, lds, s, p);
    else hipLaunchKernelGGL((conv_kernel<BMT, BN, WGM, WGN, NBUF, 1>), grid, block, lds, s, p);
}

// The 256 x 256 kernel needs 144 KiB of LDS, which a kernel has to ask for
struct BigTileInfo { int n_cu; bool lds_ok; };
BigTileInfo query_big_tile()
{
    BigTileInfo b{256, false};
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) {
        if (prop.multiProcessorCount > 0) b.n_cu = prop.multiProcessorCount;
        b.lds_ok =
            hipFuncSetAttribute((const void*)conv_kernel<256, 256, 2, 4, 2, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds) == hipSuccess &&
            hipFuncSetAttribute((const void*)conv_kernel<256, 256, 2, 4, 2, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, kBigLds) == hipSuccess;
    }
    (void)hipGetLastError();
    return b;
}

}  // namespace

hipError_t launch_conv_fast(const FastConvParams& p0, int epi, int n_active, hipStream_t s, int* stat_rows)
{
    int rows_dummy = 0;
    int& srows = stat_rows ? *stat_rows : rows_dummy;          // rows per statistics entry = rows per tile of the kernel
    if (n_active < 1) return hipSuccess;
    FastConvParams p = p0;
    p.n_active = n_active;
    if (p.C % 64 != 0 || p.N % 64 != 0) return hipErrorInvalidValue;
    // wide images with at most 128 channels in and out: the patch kernel (tiles are whole rows of one image)
    if ((p.W == 16 || p.W == 32) && p.C <= 128 && p.N <= 128 && p.R == p.S && p.R <= 3 && 2 * p.pad == p.R - 1 &&
        (p.H * p.W) % 256 == 0 && p.M % 256 == 0 && p.tile_hint != 2) {
        const int bn = (p.N % 128 == 0) ? 128 : 64;
        const dim3 block(256);
#define HADFL_PATCH(IW_, BN_, WGM_, TPS_, BMT_) do { \
            constexpr size_t loop_lds = (size_t)(BMT_ / IW_ + 2) * kPatchRowBytes<IW_> + (size_t)TPS_ * BN_ * 72 * 2; \
            constexpr size_t stat_lds = kStatLdsBytes<BN_ / (4 / WGM_) / 32, WGM_, 4 / WGM_>; \
            constexpr size_t lds = loop_lds > stat_lds ? loop_lds : stat_lds; \
            static const bool ok = hipFuncSetAttribute((const void*)conv_patch_kernel<IW_, BN_, WGM_, 0, TPS_, BMT_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess && \
                                   hipFuncSetAttribute((const void*)conv_patch_kernel<IW_, BN_, WGM_, 1, TPS_, BMT_>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) == hipSuccess; \
            if (!ok) return hipErrorInvalidValue; \
            const dim3 grid(die_grid((long long)(p.M / BMT_) * (p.N / bn) * n_active)); \
            srows = BMT_; \
            if (epi == 0) hipLaunchKernelGGL((conv_patch_kernel<IW_, BN_, WGM_, 0, TPS_, BMT_>), grid, block, lds, s, p); \
            else hipLaunchKernelGGL((conv_patch_kernel<IW_, BN_, WGM_, 1, TPS_, BMT_>), grid, block, lds, s, p); } while (0)
        // 128 output channels: waves 2 x 2; 64: waves 4 x 1
        // 32-pixel rows, 64 channels: 128-pixel tiles, four workgroups per compute unit (a tile's nine steps are too
        // short to hide its own patch load and stores: 10 % faster than 256-pixel tiles with two).  16-pixel rows, 64
        // channels: a whole filter row of weights per step where the filter has three (3-6 % faster); 128-pixel tiles
        // measured no different there, nor with 128 channels.
        if (p.W == 32 && bn == 128) HADFL_PATCH(32, 128, 2, 1, 256);
        else if (p.W == 32) HADFL_PATCH(32, 64, 4, 1, 128);
        else if (bn == 128) HADFL_PATCH(16, 128, 2, 1, 256);
        else if (p.R == 3 && p.S == 3) HADFL_PATCH(16, 64, 4, 3, 256);
        else HADFL_PATCH(16, 64, 4, 1, 256);
#undef HADFL_PATCH
        return hipGetLastError();
    }
    if (p.N % 256 == 0) {
        // One 256 x 256 workgroup per compute unit at a time: worth it when the last round of workgroups is nearly full.
        static const BigTileInfo big = query_big_tile();     // once per process (one GPU per process)
        const long long blocks = (long long)((p.M + 255) / 256) * (p.N / 256) * n_active;
        const long long rounds = (blocks + big.n_cu - 1) / big.n_cu;
        if (big.lds_ok && (p.tile_hint == 1 || blocks * 5 >= rounds * big.n_cu * 4)) {
            srows = 256;
            launch_conv_t<256, 256, 2, 4, 2>(p, epi, n_active, s);
            return hipGetLastError();
        }
    }
    const int bn = (p.N % 128 == 0) ? 128 : 64;
    // tall tiles halve the weight traffic and double the MFMA work per barrier; use them when they still fill the chip.
    // Not on layers that could have had 256 x 256 tiles: where those do not fill their last round, 128 x 128 tiles
    // measured faster than 256 x 128 at every count of active replicas.
    const bool tall = p.N % 256 != 0 && (long long)(p.M / 256) * (p.N / bn) * n_active >= 512;
    srows = tall ? 256 : 128;
    if (bn == 128) {
        if (tall) launch_conv_t<256, 128, 2, 2, 1>(p, epi, n_active, s);
        else launch_conv_t<128, 128, 2, 2, 1>(p, epi, n_active, s);
    } else {
        if (tall) launch_conv_t<256, 64, 2, 2, 1>(p, epi, n_active, s);
        else launch_conv_t<128, 64, 2, 2, 1>(p, epi, n_active, s);
    }
    return hipGetLastError();
}

hipError_t launch_wgrad_fast(const FastWgradParams& p0, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    FastWgradParams p = p0;
    p.n_active = n_active;
    if (p.C % 8 != 0 || p.N % 64 != 0) return hipErrorInvalidValue;
    // wide images with at most 128 channels in and out: all taps from one patch
    const bool wide = (p.W == 16 || p.W == 32) && p.C <= 128 && p.N <= 128 && !p.perm;
    const bool eight = p.W == 8 && p.H % 4 == 0;             // (the kernel walks pixels in memory order: no position table)
    if ((wide || eight) && p.C % 64 == 0 && p.R == 3 && p.S == 3 && p.pad == 1 &&
        (p.H * p.W) % 32 == 0 && p.K % 32 == 0 && (p.splits == 1 || p.kchunk % 32 == 0) && p.M == 9 * p.C + (p.has_bias ? 1 : 0) &&
        p.tile_hint != 2) {
        const dim3 grid(die_grid((long long)(p.C / 64) * (p.N / 64) * p.splits * n_active));
        if (p.W == 8) {
            constexpr size_t lds = 2 * ((size_t)6 * 10 + 32) * 192;
            hipLaunchKernelGGL(wgrad_taps_kernel<8>, grid, dim3(256), lds, s, p);
        } else if (p.W == 32) {
            constexpr size_t lds = 2 * ((size_t)3 * 34 + 32) * 192;
            hipLaunchKernelGGL(wgrad_taps_kernel<32>, grid, dim3(256), lds, s, p);
        } else {
            constexpr size_t lds = 2 * ((size_t)4 * 18 + 32) * 192;
            hipLaunchKernelGGL(wgrad_taps_kernel<16>, grid, dim3(256), lds, s, p);
        }
        return hipGetLastError();
    }
    // 256-row tiles (and 256 columns where the layer has them) when the launch still fills the chip
    static const BigTileInfo big = query_big_tile();
    // Only for long contractions: with few pixels per weight (the deep layers) the kernel's time is in the epilogue
    // (gradient store or fused update), which the smaller tiles overlap with other workgroups' K loops -- measured 5-30 %
    // faster there at every count of active replicas.
    int bmt = 128;
    const bool long_k = p.tile_hint == 1 || p.K >= 4096;
    if (long_k && p.N % 256 == 0) {
        const long long blocks = (long long)((p.M + 255) / 256) * (p.N / 256) * p.splits * n_active;
        const long long rounds = (blocks + big.n_cu - 1) / big.n_cu;
        if (p.tile_hint == 1 || blocks * 5 >= rounds * big.n_cu * 4) bmt = 256;
    } else if (long_k && p.N % 128 == 0) {
        if (p.tile_hint == 1 || (long long)((p.M + 255) / 256) * (p.N / 128) * p.splits * n_active >= 2LL * big.n_cu) bmt = 256;
    }
    const int bkt = bmt == 256 && p.N % 256 == 0 ? 64 : 32;
    // position-sorted contraction: a slab must hold a single position
    if (p.perm && (p.B % bkt != 0 || (p.splits > 1 && p.kchunk % bkt != 0))) return hipErrorInvalidValue;
    if (bmt == 256 && p.N % 256 == 0) {
        static const bool lds_ok = hipFuncSetAttribute((const void*)wgrad_kernel<256, 256, 2, 4, 64>,
                                                       hipFuncAttributeMaxDynamicSharedMemorySize, kBigWgradLds) == hipSuccess;
        if (!lds_ok) return hipErrorInvalidValue;
        const dim3 grid(die_grid((long long)((p.M + 255) / 256) * (p.N / 256) * p.splits * n_active));
        hipLaunchKernelGGL((wgrad_kernel<256, 256, 2, 4, 64>), grid, dim3(512), kBigWgradLds, s, p);
    } else if (bmt == 256 && p.N % 128 == 0) {
        constexpr size_t lds = 2 * 32 * ((256 + 32) * 2 + (128 + 32) * 2);
        const dim3 grid(die_grid((long long)((p.M + 255) / 256) * (p.N / 128) * p.splits * n_active));
        hipLaunchKernelGGL((wgrad_kernel<256, 128, 2, 2, 32>), grid, dim3(256), lds, s, p);
    } else if (bmt == 128 && p.N % 128 == 0) {
        constexpr size_t lds = 2 * 32 * ((128 + 32) * 2 + (128 + 32) * 2);
        const dim3 grid(die_grid((long long)((p.M + 127) / 128) * (p.N / 128) * p.splits * n_active));
        hipLaunchKernelGGL((wgrad_kernel<128, 128, 2, 2, 32>), grid, dim3(256), lds, s, p);
    } else if (bmt == 128) {
        constexpr size_t lds = 2 * 32 * ((128 + 32) * 2 + (64 + 32) * 2);
        const dim3 grid(die_grid((long long)((p.M + 127) / 128) * (p.N / 64) * p.splits * n_active));
        hipLaunchKernelGGL((wgrad_kernel<128, 64, 2, 2, 32>), grid, dim3(256), lds, s, p);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_weight_prep(const WeightPrepParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    if (p.C % 64 != 0 || p.N % 64 != 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.C / 64), (unsigned)(p.taps * (p.N / 64)), (unsigned)n_active), block(256);
    hipLaunchKernelGGL(weight_prep_kernel, grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace hadfl
