// fp32 kernels for the regular convolution layers of the fp32 configuration (3x3-style "same" convolutions, stride 1,
// input channels a multiple of 32, output channels a multiple of 64): forward and data gradient of every local step
// (paper Sec. 2.1).  Same plan as the bf16 kernels of conv_bf16_fast.hip, in fp32 on v_mfma_f32_32x32x2_f32:
//   * the weights are kept as two fp32 matrices per layer, refreshed from the master before every forward pass,
//       Wf[co][(tap, ci)]  and  Wb[ci][(flipped tap, co)],  both K-contiguous, so forward and data gradient are the SAME
//       kernel (a stride-1 data gradient is a convolution of dY with the flipped, transposed filter);
//   * a thread's pixel offset and its tap-validity mask are fixed; per slab only a wave-uniform tap delta is added;
//   * K is walked in slabs of 32 floats: eight neighbouring lanes load the full 128-byte line a row contributes, rows sit
//     in LDS at a 144-byte pitch (conflict-free 16-byte reads);
//   * the MFMA takes ONE float per lane and operand: lane (row, h = lane / 32) supplies contraction index h of the two.
//     Which two indices an instruction multiplies is free as long as both operands agree, so instruction t of a slab takes
//     k = t from the lanes of half 0 and k = 16 + t from half 1: a lane's 16 values of a slab are contiguous and arrive
//     with four 16-byte LDS reads (the generic kernel issues one 4-byte read per instruction and operand);
//   * operands are swapped (C^T = B^T A^T): 4 consecutive output channels per lane, 16-byte stores.
#include "train_kernels.h"
#include "conv_stats.h"

namespace hadfl {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
using conv_stats::store_column_stats;
using conv_stats::kStatLdsBytes;

// die d (workgroup i runs on die i % 8) takes the consecutive logical items [d * chunk, (d + 1) * chunk)
constexpr int kDies = 8;
__device__ __forceinline__ unsigned logical_block()
{
    const unsigned chunk = gridDim.x / kDies;
    return (blockIdx.x % kDies) * chunk + blockIdx.x / kDies;
}
inline unsigned die_grid(long long items) { return (unsigned)((items + kDies - 1) / kDies * kDies); }

__device__ __forceinline__ u4 ldg16(const char* base, unsigned off) { return *reinterpret_cast<const u4*>(base + off); }

// GEMM row m -> pixel index and the set of taps inside the image.  With a position table (p.perm) row ps * B + b is image
// b at pixel position perm[ps] (positions sorted by their tap sets); without one rows are pixels in memory order.
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
// taps some row of the tile [m0, m0 + rows) can reach
__device__ __forceinline__ unsigned tile_taps(const FastConvParams& p, int m0, int rows)
{
    const unsigned all = (p.R * p.S >= 32) ? 0xffffffffu : ((1u << (p.R * p.S)) - 1u);
    if (!p.perm) return all;
    const int last = min(m0 + rows, p.M) - 1;
    unsigned u = 0;
    for (int ps = m0 / p.B; ps <= last / p.B; ++ps) u |= p.posmask[ps];
    return u & all;
}

// Tile BMT x BN, WGM x WGN waves (wave tile BMT/WGM x BN/WGN), one LDS buffer: the next slab waits in registers while
// the current one is multiplied, two barriers per slab.  EPI 0: + bias, optional ReLU;  EPI 1: optional mask, optional
// accumulate.  p.a, p.wmat, p.out, p.mask are fp32 here (wmat_rep in floats).
template <int BMT, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(WGM * WGN * 64, 2) void conv_f32_kernel(FastConvParams p)
{
    constexpr int NT = WGM * WGN * 64;
    constexpr int BK = 32, PITCH = 144;                       // floats per slab row; LDS bytes per row
    constexpr int TM = BMT / WGM / 32, TN = BN / WGN / 32;
    constexpr int NQA = BMT * 8 / NT, NQB = BN * 8 / NT;      // 16-byte slots per thread: rows x 8 groups of 4 k
    static_assert(NQA >= 1 && NQB >= 1 && TM >= 1 && TN >= 1, "tile too small for the thread count");
    constexpr unsigned A_BUF = BMT * PITCH;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* const sAc = smem;                           // [BMT][PITCH]
    char* const sBc = smem + A_BUF;                   // [BN][PITCH]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WGN, wn = wave % WGN;
    // logical item = (slot, column tile, row tile), row tiles fastest
    const unsigned tiles_m = (unsigned)(p.M + BMT - 1) / BMT, tiles_n = (unsigned)p.N / BN;
    const unsigned item = logical_block();
    if (item >= tiles_m * tiles_n * (unsigned)p.n_active) return;
    const int rep = p.order[item / (tiles_m * tiles_n)];
    const int m0 = (int)(item % tiles_m) * BMT, n0 = (int)((item / tiles_m) % tiles_n) * BN;
    const char* abase = (const char*)p.a + (long long)rep * p.a_rep * 4;
    const char* wbase = (const char*)p.wmat + (long long)rep * p.wmat_rep * 4;

    unsigned aoff[NQA], boff[NQB], sa_st[NQA], sb_st[NQB], tapmask[NQA];
#pragma unroll
    for (int q = 0; q < NQA; ++q) {
        const int i = tid + q * NT;
        const int arow = i >> 3, kq = i & 7;
        const RowGeo g = row_geo(p, m0 + arow);
        tapmask[q] = g.tapmask;
        aoff[q] = (unsigned)(g.pix * p.C + kq * 4) * 4u;
        sa_st[q] = (unsigned)(arow * PITCH + kq * 16);
    }
#pragma unroll
    for (int q = 0; q < NQB; ++q) {
        const int i = tid + q * NT;
        boff[q] = (unsigned)((n0 + (i >> 3)) * p.K + (i & 7) * 4) * 4u;
        sb_st[q] = (unsigned)((i >> 3) * PITCH + (i & 7) * 16);
    }
    // lane (row, h) reads the 16 floats k = 16 h .. 16 h + 15 of its row
    const unsigned a_rd = (unsigned)((wm * (BMT / WGM) + (lane & 31)) * PITCH + (lane >> 5) * 64);
    const unsigned b_rd = (unsigned)((wn * (BN / WGN) + (lane & 31)) * PITCH + (lane >> 5) * 64);

    // slabs: (tap, 32 channels) for the taps of this tile, taps ascending
    const unsigned taps = tile_taps(p, m0, BMT);
    const int nslab = __builtin_popcount(taps) * (p.C / BK);
    unsigned taps_left = taps;
    int tap = taps ? __builtin_ctz(taps) : 0, c0 = 0;
    u4 ra[NQA], rb[NQB];
    auto load_tiles = [&]() {
        const int r = tap / p.S, s = tap - r * p.S;
        const int delta = (((r - p.pad) * p.W + (s - p.pad)) * p.C + c0) * 4;       // bytes, may be negative
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            u4 v = {0u, 0u, 0u, 0u};
            if ((tapmask[q] >> tap) & 1u) v = ldg16(abase, aoff[q] + (unsigned)delta);
            ra[q] = v;
        }
        const unsigned kb = (unsigned)(tap * p.C + c0) * 4u;
#pragma unroll
        for (int q = 0; q < NQB; ++q) rb[q] = ldg16(wbase, boff[q] + kb);
        c0 += BK;
        if (c0 == p.C) {
            c0 = 0;
            taps_left &= taps_left - 1u;                 // drop the tap just finished
            tap = taps_left ? __builtin_ctz(taps_left) : 0;
        }
    };
    auto store_tiles = [&]() {
#pragma unroll
        for (int q = 0; q < NQA; ++q) *reinterpret_cast<u4*>(sAc + sa_st[q]) = ra[q];
#pragma unroll
        for (int q = 0; q < NQB; ++q) *reinterpret_cast<u4*>(sBc + sb_st[q]) = rb[q];
    };

    f16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto compute = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f4 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const f4*>(sAc + a_rd + i * 32 * PITCH + q * 16);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const f4*>(sBc + b_rd + j * 32 * PITCH + q * 16);
#pragma unroll
            for (int e = 0; e < 4; ++e)
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TN; ++j)      // operands swapped: the accumulator holds the transposed tile
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(b[j][e], a[i][e], acc[i][j], 0, 0, 0);
        }
    };

    if (nslab > 0) {
        load_tiles();
        for (int t = 0; t < nslab; ++t) {
            __syncthreads();                               // every wave is done reading the previous slab
            store_tiles();
            __syncthreads();
            if (t + 1 < nslab) load_tiles();
            compute();
        }
    }

    // ---- epilogue: lane holds output row (lane & 31) and channels 8*g + 4*(lane >> 5) + {0..3}, g = 0..3 ----
    float* obase = (float*)p.out + (long long)rep * p.out_rep;
    const float* bias = (EPI == 0 && p.bias) ? p.bias + (long long)rep * p.bias_rep : nullptr;
    const float* mask = (EPI == 1 && p.mask) ? (const float*)p.mask + (long long)rep * p.mask_rep : nullptr;
    const bool stats = EPI == 0 && p.stat != nullptr;         // per-channel sums of the outputs for a batch norm that follows
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
                const long long o = (long long)pix * p.N + n;
                f4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                f4 sh = {0.f, 0.f, 0.f, 0.f};                  // what the statistics are centred on: the bias
                if (EPI == 0) {
                    if (bias) { sh = *reinterpret_cast<const f4*>(bias + n); v += sh; }
                    if (p.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                } else {
                    if (mask) {
                        const f4 mk = *reinterpret_cast<const f4*>(mask + o);
#pragma unroll
                        for (int e = 0; e < 4; ++e) if (!(mk[e] > 0.f)) v[e] = 0.f;
                    }
                    if (p.accumulate) v += *reinterpret_cast<const f4*>(obase + o);
                }
                *reinterpret_cast<f4*>(obase + o) = v;
                if (stats) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) { const float f = v[e] - sh[e]; ss[j][4 * g + e] += f; qq[j][4 * g + e] += f * f; }
                }
            }
        }
    }
    if (stats) {                                              // (the launcher asks for the larger of the K loop's LDS and kStatLdsBytes)
        __syncthreads();                                      // every wave is past its last operand read
        const int slot = (int)(item / (tiles_m * tiles_n));
        store_column_stats<TN, WGM, WGN>(ss, qq, reinterpret_cast<float*>(smem), wave, lane, p.stat + (long long)slot * p.stat_rep,
                                         m0 / BMT, n0 + wn * (BN / WGN), p.N);
    }
}

// fp32 master W[tap][ci][co] -> Wf[co][tap*C + ci] and Wb[ci][(T-1-tap)*N + co], both fp32.  A workgroup handles one tap
// and a 64 x 64 (ci, co) tile.
__global__ __launch_bounds__(256) void weight_prep_f32_kernel(WeightPrepF32Params p)
{
    __shared__ float tile[64][65];
    const int rep = p.order[blockIdx.z];
    const int taps = p.taps;
    const int tap = blockIdx.y % taps, cot = blockIdx.y / taps;
    const int ci0 = blockIdx.x * 64, co0 = cot * 64;
    const float* w = p.w + (long long)rep * p.w_rep + ((long long)tap * p.C) * p.N;
    float* wf = p.wf + (long long)rep * p.wcopy_rep;
    float* wb = p.wb + (long long)rep * p.wcopy_rep;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int K = taps * p.C, Kb = taps * p.N;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int ci = ci0 + ty + 4 * r;
        float v = 0.f;
        if (ci < p.C) {
            v = w[(long long)ci * p.N + co0 + tx];
            wb[(long long)ci * Kb + (taps - 1 - tap) * p.N + co0 + tx] = v;
        }
        tile[ty + 4 * r][tx] = v;
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int co = co0 + ty + 4 * r;
        if (ci0 + tx < p.C) wf[(long long)co * K + tap * p.C + ci0 + tx] = tile[tx][ty + 4 * r];
    }
}

template <int BMT, int BN, int WGM, int WGN>
void launch_t(const FastConvParams& p, int epi, int n_active, hipStream_t s)
{
    constexpr size_t loop_lds = (size_t)(BMT + BN) * 144, stat_lds = kStatLdsBytes<BN / WGN / 32, WGM, WGN>;
    constexpr size_t lds = loop_lds > stat_lds ? loop_lds : stat_lds;
    const dim3 grid(die_grid((long long)((p.M + BMT - 1) / BMT) * (p.N / BN) * n_active)), block(WGM * WGN * 64);
    if (epi == 0) hipLaunchKernelGGL((conv_f32_kernel<BMT, BN, WGM, WGN, 0>), grid, block, lds, s, p);
    else hipLaunchKernelGGL((conv_f32_kernel<BMT, BN, WGM, WGN, 1>), grid, block, lds, s, p);
}

}  // namespace

hipError_t launch_conv_f32_fast(const FastConvParams& p0, int epi, int n_active, hipStream_t s, int* stat_rows)
{
    if (n_active < 1) return hipSuccess;
    FastConvParams p = p0;
    p.n_active = n_active;
    if (p.C % 32 != 0 || p.N % 64 != 0) return hipErrorInvalidValue;
    // tall tiles halve the weight traffic and double the MFMA work per barrier; use them when they still fill the chip
    const int bn = (p.N % 128 == 0) ? 128 : 64;
    const bool tall = p.tile_hint == 1 || (long long)(p.M / 256) * (p.N / bn) * n_active >= 512;
    if (stat_rows) *stat_rows = tall ? 256 : 128;             // rows per statistics entry = rows per tile
    if (bn == 128) {
        if (tall) launch_t<256, 128, 2, 2>(p, epi, n_active, s);
        else launch_t<128, 128, 2, 2>(p, epi, n_active, s);
    } else {
        if (tall) launch_t<256, 64, 2, 2>(p, epi, n_active, s);
        else launch_t<128, 64, 2, 2>(p, epi, n_active, s);
    }
    return hipGetLastError();
}

hipError_t launch_weight_prep_f32(const WeightPrepF32Params& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    if (p.N % 64 != 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((p.C + 63) / 64), (unsigned)(p.taps * (p.N / 64)), (unsigned)n_active), block(256);
    hipLaunchKernelGGL(weight_prep_f32_kernel, grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace hadfl
