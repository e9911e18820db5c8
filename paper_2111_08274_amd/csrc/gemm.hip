// Grouped implicit-GEMM kernel for convolutions and dense layers on the fp32 matrix cores of gfx950
// (v_mfma_f32_32x32x2_f32), forward, data gradient and weight gradient, for all active replicas in one launch.
//
// Tiling: a workgroup of WM x WN wavefronts owns a BM x BN tile of C; K is walked in slabs of 16 staged through
// LDS (double buffered, one barrier per slab) as A[k][m] and B[k][n], so that the MFMA operand reads
// (lane -> m or n, lane/32 -> k) are unit-stride.  Operands whose memory order runs along K are transposed on
// the way into LDS.  The im2col matrices are never materialised: loaders compute addresses from the geometry.
#include <cstdint>
#include "train_kernels.h"

namespace hadfl {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;

__device__ __forceinline__ f4 ld4(const float* p) { return *reinterpret_cast<const f4*>(p); }

template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(64 * WM * WN) void igemm_kernel(GemmParams p)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    constexpr int A_SLOTS = BM * BK / 4, B_SLOTS = BN * BK / 4;
    constexpr int NQA = (A_SLOTS + NT - 1) / NT, NQB = (B_SLOTS + NT - 1) / NT;
    static_assert(TM >= 1 && TN >= 1, "tile too small for the wave grid");
    // Operands read along K are staged as slot i = (row i / 4, k-group i % 4): four neighbouring lanes read the 64
    // contiguous bytes one row contributes to a slab.  The +4 pitch keeps their transposing LDS writes (4 k-rows x
    // 16 columns per wave instruction) in distinct banks.
    __shared__ __attribute__((aligned(16))) float sA[2][BK][BM + 4];
    __shared__ __attribute__((aligned(16))) float sB[2][BK][BN + 4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    // One-dimensional grid of 8 * chunk workgroups.  Workgroups are handed to the eight dies in turn (workgroup i runs
    // on die i % 8, each die with its own L2); die d takes the consecutive logical items [d * chunk, (d + 1) * chunk),
    // item = (slot, split or class, tile), so the tiles of one replica meet in one L2.
    const unsigned chunk = gridDim.x / 8u;
    const unsigned item = (blockIdx.x % 8u) * chunk + blockIdx.x / 8u;
    const unsigned tiles = (unsigned)(p.tiles_m * p.tiles_n);
    if (item >= tiles * (unsigned)p.grid_y * (unsigned)p.n_active) return;
    const int slot = (int)(item / (tiles * (unsigned)p.grid_y));
    const int by = (int)((item / tiles) % (unsigned)p.grid_y);
    const int bx = (int)(item % tiles);
    const int rep = p.order[slot];
    const int tile_m = bx / p.tiles_n, tile_n = bx % p.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int split = by;
    const int kbeg = (MODE == kDgrad) ? 0 : split * p.kchunk;

    // activation-side base for this replica (the data set is indexed through the batch cursor)
    const float* abase;
    if (p.cursor) {
        const long long first = (p.cursor[rep] * (long long)p.batch) % p.n_samples;
        abase = p.a + ((long long)rep * p.n_samples + first) * p.sample_sz;
    } else {
        abase = p.a + (long long)rep * p.a_rep;
    }
    const float* wbase = p.w + (long long)rep * p.w_rep;

    // kDgrad: an input pixel (y, x) only receives taps with r = (y + pad) mod stride (likewise s), so the pixels are
    // split into stride*stride classes by (y mod stride, x mod stride); a class is a dense GEMM over its own tap list
    // and no multiply-add is spent on taps that never contribute.  `by` is the class (1 class for stride 1).
    int d_ph = 0, d_pw = 0, d_r0 = 0, d_s0 = 0, d_ns = p.S, d_hc = p.H, d_wc = p.W, d_m = p.M;
    int kend = min(p.K, kbeg + p.kchunk);
    if (MODE == kDgrad) {
        d_ph = by / p.stride; d_pw = by % p.stride;
        d_hc = (p.H - d_ph + p.stride - 1) / p.stride; d_wc = (p.W - d_pw + p.stride - 1) / p.stride;
        d_r0 = (d_ph + p.pad) % p.stride; d_s0 = (d_pw + p.pad) % p.stride;
        const int nr = d_r0 < p.R ? (p.R - d_r0 + p.stride - 1) / p.stride : 0;
        d_ns = d_s0 < p.S ? (p.S - d_s0 + p.stride - 1) / p.stride : 0;
        d_m = p.B * d_hc * d_wc;
        kend = nr * d_ns * p.Cout;
        if (m0 >= d_m) return;
    }
    // ---------------- per-thread, loop-invariant parts of the operand addresses ----------------
    // kFwd / kDgrad: A is read along K for one fixed row m.
    int a_b[NQA], a_y[NQA], a_x[NQA]; bool a_ok[NQA];
    // kWgrad: A is read along M for a fixed group of 4 rows m..m+3.
    int wa_m = 0, wa_r = 0, wa_s = 0, wa_c = 0;
    if (MODE == kWgrad) {
        wa_m = m0 + (tid % (BM / 4)) * 4;
        const int tap = wa_m / p.Cin;
        wa_c = wa_m - tap * p.Cin;
        wa_r = tap / p.S; wa_s = tap - wa_r * p.S;
    } else {
        const int hw = (MODE == kFwd) ? p.Ho * p.Wo : d_hc * d_wc;
        const int ww = (MODE == kFwd) ? p.Wo : d_wc;
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int a_m = m0 + ((tid + q * NT) >> 2);
            a_ok[q] = a_m < ((MODE == kFwd) ? p.M : d_m);
            a_b[q] = a_m / hw;
            const int rem = a_m - a_b[q] * hw;
            a_y[q] = rem / ww; a_x[q] = rem - a_y[q] * ww;
            if (MODE == kDgrad) { a_y[q] = a_y[q] * p.stride + d_ph; a_x[q] = a_x[q] * p.stride + d_pw; }
        }
    }
    const bool fastA = (MODE == kFwd) ? (p.Cin % BK == 0) : (MODE == kDgrad) ? (p.Cout % BK == 0) : (p.Cin % 4 == 0);
    const bool vecN = (p.N % 4 == 0);

    f4 ra[NQA], rb[NQB];

    auto load_tiles = [&](int k0) {
        // ------------------------------ A ------------------------------
        if (MODE == kFwd) {
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
                const int i = tid + q * NT;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (i < A_SLOTS) {
                    const int kq = i & 3;
                    if (fastA) {
                        const int tap = k0 / p.Cin, c0 = k0 - tap * p.Cin;
                        const int r = tap / p.S, s = tap - r * p.S;
                        const int yy = a_y[q] * p.stride - p.pad + r, xx = a_x[q] * p.stride - p.pad + s;
                        if (a_ok[q] && yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                            v = ld4(abase + (((long long)a_b[q] * p.H + yy) * p.W + xx) * p.Cin + c0 + kq * 4);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int k = k0 + kq * 4 + j;
                            if (a_ok[q] && k < kend) {
                                const int tap = k / p.Cin, c = k - tap * p.Cin;
                                const int r = tap / p.S, s = tap - r * p.S;
                                const int yy = a_y[q] * p.stride - p.pad + r, xx = a_x[q] * p.stride - p.pad + s;
                                if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                                    v[j] = abase[(((long long)a_b[q] * p.H + yy) * p.W + xx) * p.Cin + c];
                            }
                        }
                    }
                }
                ra[q] = v;
            }
        } else if (MODE == kDgrad) {
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
                const int i = tid + q * NT;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (i < A_SLOTS) {
                    const int kq = i & 3;
                    if (fastA) {
                        const int tap = k0 / p.Cout, c0 = k0 - tap * p.Cout;
                        const int ir = tap / d_ns, is = tap - ir * d_ns;
                        const int ty = a_y[q] + p.pad - (d_r0 + ir * p.stride), tx = a_x[q] + p.pad - (d_s0 + is * p.stride);
                        const int yo = ty / p.stride, xo = tx / p.stride;      // exact: the class fixes the residue
                        if (a_ok[q] && ty >= 0 && tx >= 0 && yo < p.Ho && xo < p.Wo)
                            v = ld4(abase + (((long long)a_b[q] * p.Ho + yo) * p.Wo + xo) * p.Cout + c0 + kq * 4);
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const int k = k0 + kq * 4 + j;
                            if (a_ok[q] && k < kend) {
                                const int tap = k / p.Cout, c = k - tap * p.Cout;
                                const int ir = tap / d_ns, is = tap - ir * d_ns;
                                const int ty = a_y[q] + p.pad - (d_r0 + ir * p.stride), tx = a_x[q] + p.pad - (d_s0 + is * p.stride);
                                const int yo = ty / p.stride, xo = tx / p.stride;
                                if (ty >= 0 && tx >= 0 && yo < p.Ho && xo < p.Wo)
                                    v[j] = abase[(((long long)a_b[q] * p.Ho + yo) * p.Wo + xo) * p.Cout + c];
                            }
                        }
                    }
                }
                ra[q] = v;
            }
        } else {   // kWgrad: A[m = (tap, ci) | bias row][k = (b, yo, xo)], contiguous along m
            const int mw = p.R * p.S * p.Cin;    // rows that are weights; row mw (if present) collects the bias gradient
#pragma unroll
            for (int q = 0; q < NQA; ++q) {
                const int i = tid + q * NT;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (i < A_SLOTS) {
                    const int k = k0 + i / (BM / 4);
                    if (k < kend) {
                        int b, yo, xo;
                        if (p.hw_shift >= 0) {
                            b = k >> p.hw_shift;
                            const int rem = k & ((1 << p.hw_shift) - 1);
                            yo = rem >> p.w_shift; xo = rem & ((1 << p.w_shift) - 1);
                        } else {
                            const int hw = p.Ho * p.Wo;
                            b = k / hw;
                            const int rem = k - b * hw;
                            yo = rem / p.Wo; xo = rem - yo * p.Wo;
                        }
                        if (fastA) {
                            if (wa_m < mw) {
                                const int yy = yo * p.stride - p.pad + wa_r, xx = xo * p.stride - p.pad + wa_s;
                                if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                                    v = ld4(abase + (((long long)b * p.H + yy) * p.W + xx) * p.Cin + wa_c);
                            } else if (wa_m == mw && p.has_bias) {
                                v[0] = 1.f;
                            }
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int m = wa_m + j;
                                if (m < mw) {
                                    const int tap = m / p.Cin, c = m - tap * p.Cin;
                                    const int r = tap / p.S, s = tap - r * p.S;
                                    const int yy = yo * p.stride - p.pad + r, xx = xo * p.stride - p.pad + s;
                                    if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                                        v[j] = abase[(((long long)b * p.H + yy) * p.W + xx) * p.Cin + c];
                                } else if (m == mw && p.has_bias) {
                                    v[j] = 1.f;
                                }
                            }
                        }
                    }
                }
                ra[q] = v;
            }
        }
        // ------------------------------ B ------------------------------
        if (MODE == kDgrad) {   // B[k = (tap, co)][n = ci] = W[tap][ci][co], contiguous along k
            const bool fastB = (p.Cout % BK == 0);
#pragma unroll
            for (int q = 0; q < NQB; ++q) {
                const int i = tid + q * NT;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (i < B_SLOTS) {
                    const int n = n0 + (i >> 2), kq = i & 3;
                    if (n < p.N) {
                        if (fastB) {
                            const int t = k0 / p.Cout, c0 = k0 - t * p.Cout;
                            const int ir = t / d_ns, is = t - ir * d_ns;
                            const int tap = (d_r0 + ir * p.stride) * p.S + d_s0 + is * p.stride;
                            v = ld4(wbase + ((long long)tap * p.Cin + n) * p.Cout + c0 + kq * 4);
                        } else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                const int k = k0 + kq * 4 + j;
                                if (k < kend) {
                                    const int t = k / p.Cout, c = k - t * p.Cout;
                                    const int ir = t / d_ns, is = t - ir * d_ns;
                                    const int tap = (d_r0 + ir * p.stride) * p.S + d_s0 + is * p.stride;
                                    v[j] = wbase[((long long)tap * p.Cin + n) * p.Cout + c];
                                }
                            }
                        }
                    }
                }
                rb[q] = v;
            }
        } else {                // B[k][n] row-major with pitch N: the weights (kFwd) or dY (kWgrad)
            const float* bsrc = (MODE == kFwd) ? wbase : (p.dy + (long long)rep * p.dy_rep);
#pragma unroll
            for (int q = 0; q < NQB; ++q) {
                const int i = tid + q * NT;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (i < B_SLOTS) {
                    const int n = n0 + (i % (BN / 4)) * 4, k = k0 + i / (BN / 4);
                    if (k < kend) {
                        const float* src = bsrc + (long long)k * p.N + n;
                        if (vecN) { if (n < p.N) v = ld4(src); }
                        else {
#pragma unroll
                            for (int j = 0; j < 4; ++j) if (n + j < p.N) v[j] = src[j];
                        }
                    }
                }
                rb[q] = v;
            }
        }
    };

    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int i = tid + q * NT;
            if (i < A_SLOTS) {
                if (MODE == kWgrad) {
                    *reinterpret_cast<f4*>(&sA[buf][i / (BM / 4)][(i % (BM / 4)) * 4]) = ra[q];
                } else {
                    const int ml = i >> 2, kq = i & 3;
#pragma unroll
                    for (int j = 0; j < 4; ++j) sA[buf][kq * 4 + j][ml] = ra[q][j];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) {
            const int i = tid + q * NT;
            if (i < B_SLOTS) {
                if (MODE == kDgrad) {
                    const int nl = i >> 2, kq = i & 3;
#pragma unroll
                    for (int j = 0; j < 4; ++j) sB[buf][kq * 4 + j][nl] = rb[q][j];
                } else {
                    *reinterpret_cast<f4*>(&sB[buf][i / (BN / 4)][(i % (BN / 4)) * 4]) = rb[q];
                }
            }
        }
    };

    f16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int nslab = (kend - kbeg + BK - 1) / BK;
    if (nslab > 0) {
        load_tiles(kbeg);
        store_tiles(0);
    }
    __syncthreads();
    for (int t = 0; t < nslab; ++t) {
        const int buf = t & 1;
        if (t + 1 < nslab) load_tiles(kbeg + (t + 1) * BK);
#pragma unroll
        for (int kk = 0; kk < BK / 2; ++kk) {
            const int kr = kk * 2 + (lane >> 5);
            float a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = sA[buf][kr][(wm * TM + i) * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = sB[buf][kr][(wn * TN + j) * 32 + (lane & 31)];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < nslab) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue: lane holds column (lane & 31), rows 8*(v/4) + 4*(lane>>5) + v%4 ----------------
    float* obase;
    if (MODE == kWgrad && p.splits > 1)
        obase = p.out + (long long)slot * p.out_rep + (long long)split * p.out_split;
    else
        obase = p.out + (long long)rep * p.out_rep;
    const float* bias = (MODE == kFwd && p.has_bias) ? (wbase + (long long)p.K * p.N) : nullptr;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int n = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (n >= p.N) continue;
        const float bv = bias ? bias[n] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int m = m0 + (wm * TM + i) * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (m >= ((MODE == kDgrad) ? d_m : p.M)) continue;
                float r = acc[i][j][v];
                long long row = m;
                if (MODE == kDgrad && p.stride > 1) {
                    const int hw = d_hc * d_wc;
                    const int b = m / hw, rem = m - b * hw;
                    const int yy = rem / d_wc, xx = rem - yy * d_wc;
                    row = ((long long)b * p.H + yy * p.stride + d_ph) * p.W + xx * p.stride + d_pw;
                }
                float* dst = obase + row * p.N + n;
                if (MODE == kFwd) {
                    r += bv;
                    if (p.relu) r = fmaxf(r, 0.f);
                } else if (MODE == kDgrad) {
                    if (p.mask && !(p.mask[(long long)rep * p.mask_rep + row * p.N + n] > 0.f)) r = 0.f;
                    if (p.accumulate) r += *dst;
                }
                *dst = r;
            }
        }
    }
}

// out[i] = sum over splits of partial[s][i].  A workgroup covers 32 outputs with 8 lanes each: lane j adds the splits
// s = j, j+8, ... in ascending order, then the 8 partial sums are combined by a fixed butterfly (deterministic).
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, long long split_stride,
                                                            int splits, float* __restrict__ out, long long out_rep,
                                                            long long count, const int* __restrict__ order)
{
    __shared__ float red[8][32];
    const int g = blockIdx.y, rep = order[g];
    const float* src = partial + (long long)g * split_stride * splits;
    float* dst = out + (long long)rep * out_rep;
    const int el = threadIdx.x & 31, sl = threadIdx.x >> 5;
    for (long long i0 = (long long)blockIdx.x * 32; i0 < count; i0 += (long long)gridDim.x * 32) {
        const long long i = i0 + el;
        float s = 0.f;
        if (i < count)
            for (int k = sl; k < splits; k += 8) s += src[(long long)k * split_stride + i];
        red[sl][el] = s;
        __syncthreads();
        if (sl == 0 && i < count)
            dst[i] = ((red[0][el] + red[1][el]) + (red[2][el] + red[3][el])) + ((red[4][el] + red[5][el]) + (red[6][el] + red[7][el]));
        __syncthreads();
    }
}

// The same sum for counts that are a multiple of 4: one thread per 4 consecutive outputs, splits added one after another
// in ascending order with 16-byte accesses.
__global__ __launch_bounds__(256) void splitk_reduce_vec_kernel(const float* __restrict__ partial, long long split_stride,
                                                                int splits, float* __restrict__ out, long long out_rep,
                                                                long long count4, const int* __restrict__ order)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int g = blockIdx.y, rep = order[g];
    const f4* src = reinterpret_cast<const f4*>(partial + (long long)g * split_stride * splits);
    f4* dst = reinterpret_cast<f4*>(out + (long long)rep * out_rep);
    const long long stride4 = split_stride / 4;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count4; i += (long long)gridDim.x * 256) {
        f4 acc = src[i];
#pragma unroll 4
        for (int k = 1; k < splits; ++k) acc = acc + src[(long long)k * stride4 + i];
        dst[i] = acc;
    }
}

// The same sum, applied as the parameter update instead of being stored: buf = momentum*buf + g; w = w - lr*buf
// (local-update equation of Sec. 2.2).  w and buf point at the layer's parameters inside the replica rows.
__global__ __launch_bounds__(256) void splitk_reduce_update_kernel(const float* __restrict__ partial, long long split_stride,
                                                                   int splits, float* __restrict__ w, float* __restrict__ buf,
                                                                   long long row_stride, long long count4, float lr, float momentum,
                                                                   const int* __restrict__ order)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const int g = blockIdx.y, rep = order[g];
    const f4* src = reinterpret_cast<const f4*>(partial + (long long)g * split_stride * splits);
    f4* wd = reinterpret_cast<f4*>(w + (long long)rep * row_stride);
    f4* bd = buf ? reinterpret_cast<f4*>(buf + (long long)rep * row_stride) : nullptr;
    const long long stride4 = split_stride / 4;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < count4; i += (long long)gridDim.x * 256) {
        f4 acc = __builtin_nontemporal_load(src + i);              // partial sums, parameters, momentum: each touched once
#pragma unroll 4
        for (int k = 1; k < splits; ++k) acc = acc + __builtin_nontemporal_load(src + (long long)k * stride4 + i);
        if (bd) { acc = __builtin_nontemporal_load(bd + i) * momentum + acc; __builtin_nontemporal_store(acc, bd + i); }
        __builtin_nontemporal_store(__builtin_nontemporal_load(wd + i) - acc * lr, wd + i);
    }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_tile(const GemmParams& p0, int n_active, hipStream_t s)
{
    GemmParams p = p0;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    unsigned gy = (unsigned)p.splits;
    if (p.mode == kDgrad) {
        gy = (unsigned)(p.stride * p.stride);
        const int rows0 = p.B * ((p.H + p.stride - 1) / p.stride) * ((p.W + p.stride - 1) / p.stride);   // largest class
        p.tiles_m = (rows0 + BM - 1) / BM;
    }
    p.grid_y = (int)gy; p.n_active = n_active;
    const long long items = (long long)p.tiles_m * p.tiles_n * gy * n_active;
    const dim3 grid((unsigned)((items + 7) / 8 * 8)), block(64 * WM * WN);
    switch (p.mode) {
    case kFwd: hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, kFwd>), grid, block, 0, s, p); break;
    case kDgrad: hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, kDgrad>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((igemm_kernel<BM, BN, WM, WN, kWgrad>), grid, block, 0, s, p); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm(const GemmParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1 || p.M < 1 || p.N < 1) return hipSuccess;
    // tile choice: widest N tile the layer fills, tallest M tile that still leaves enough workgroups
    const int bn = p.N > 64 ? 128 : (p.N > 32 ? 64 : 32);
    const long long rows_blocks_128 = (long long)((p.M + 127) / 128) * ((p.N + bn - 1) / bn) * p.splits * n_active;
    const bool tall = p.M >= 128 && rows_blocks_128 >= 256;
    if (bn == 128) return tall ? launch_tile<128, 128, 2, 2>(p, n_active, s) : launch_tile<64, 128, 1, 4>(p, n_active, s);
    if (bn == 64) return tall ? launch_tile<128, 64, 2, 2>(p, n_active, s) : launch_tile<64, 64, 2, 2>(p, n_active, s);
    return tall ? launch_tile<128, 32, 4, 1>(p, n_active, s) : launch_tile<32, 32, 1, 1>(p, n_active, s);
}

hipError_t launch_splitk_reduce(const float* partial, long long split_stride, int splits, float* out, long long out_rep,
                                long long count, const int* order, int n_active, hipStream_t s)
{
    if (n_active < 1 || count < 1) return hipSuccess;
    if (count % 4 == 0 && split_stride % 4 == 0 && out_rep % 4 == 0 && (((uintptr_t)partial | (uintptr_t)out) & 15) == 0) {
        long long bx = (count / 4 + 255) / 256;
        if (bx > 2048) bx = 2048;
        hipLaunchKernelGGL(splitk_reduce_vec_kernel, dim3((unsigned)bx, (unsigned)n_active), dim3(256), 0, s, partial,
                           split_stride, splits, out, out_rep, count / 4, order);
        return hipGetLastError();
    }
    long long bx = (count + 31) / 32;
    if (bx > 4096) bx = 4096;
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)bx, (unsigned)n_active), dim3(256), 0, s, partial,
                       split_stride, splits, out, out_rep, count, order);
    return hipGetLastError();
}

hipError_t launch_splitk_reduce_update(const float* partial, long long split_stride, int splits, float* w, float* buf,
                                       long long row_stride, long long count, float lr, float momentum, const int* order,
                                       int n_active, hipStream_t s)
{
    if (n_active < 1 || count < 1) return hipSuccess;
    if (count % 4 != 0 || split_stride % 4 != 0 || row_stride % 4 != 0 ||
        (((uintptr_t)partial | (uintptr_t)w | (uintptr_t)buf) & 15) != 0) return hipErrorInvalidValue;
    long long bx = (count / 4 + 255) / 256;
    if (bx > 2048) bx = 2048;
    hipLaunchKernelGGL(splitk_reduce_update_kernel, dim3((unsigned)bx, (unsigned)n_active), dim3(256), 0, s, partial,
                       split_stride, splits, w, buf, row_stride, count / 4, lr, momentum, order);
    return hipGetLastError();
}

}  // namespace hadfl
