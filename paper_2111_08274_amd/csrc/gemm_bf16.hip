// Grouped implicit-GEMM kernel for the bf16 configuration: bf16 activations and activation gradients, fp32 master
// weights rounded to bf16 while they are staged, fp32 accumulation on v_mfma_f32_32x32x16_bf16 (gfx950).
//
// A workgroup of WM x WN wavefronts owns a BM x BN tile; K is walked in slabs of 32 through double-buffered LDS.
// The bf16 MFMA wants 8 consecutive k per lane, so both operands sit in LDS as [row][k] (k contiguous, rows padded
// to 40 elements = 80 bytes, which makes the 16-byte operand reads bank-conflict free).  Operands whose memory order
// already runs along k (activations in forward / data-gradient, the transposed weights in data-gradient) are copied
// 16 bytes at a time; operands that run along m or n (weights in forward, both operands of the weight gradient) are
// transposed on the way in: a thread takes two consecutive k rows of four columns and writes four 32-bit (k, k+1)
// pairs.  Layers whose channel counts do not allow the vector paths (the 3-channel input, the 10-wide classifier)
// go through a scalar fetch with the same results.
#include "train_kernels.h"

namespace hadfl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));

constexpr int BK = 32;
constexpr int LDP = 40;     // LDS row pitch in bf16 elements

__device__ __forceinline__ unsigned pack2(float lo, float hi)
{
    bf16x2 v; v[0] = (__bf16)lo; v[1] = (__bf16)hi;
    return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ unsigned pack2b(__bf16 lo, __bf16 hi)
{
    bf16x2 v; v[0] = lo; v[1] = hi;
    return __builtin_bit_cast(unsigned, v);
}

// Geometry shared by the loaders of one workgroup.
struct Geo {
    int kend;                                           // contraction length of this workgroup's problem
    int d_ph, d_pw, d_r0, d_s0, d_ns, d_hc, d_wc, d_m;  // data-gradient pixel class (see the fp32 kernel)
};

template <int MODE>
__device__ __forceinline__ float fetch_a(const GemmParams& p, const Geo& g, const void* abase, int m, int k)
{
    // value of A[m][k] as a float (0 outside the problem); abase is bf16 unless p.a_f32
    if (MODE == kFwd) {
        if (m >= p.M || k >= g.kend) return 0.f;
        const int hw = p.Ho * p.Wo;
        const int b = m / hw, rem = m - b * hw, yo = rem / p.Wo, xo = rem - yo * p.Wo;
        const int tap = k / p.Cin, c = k - tap * p.Cin, r = tap / p.S, s = tap - r * p.S;
        const int yy = yo * p.stride - p.pad + r, xx = xo * p.stride - p.pad + s;
        if (yy < 0 || yy >= p.H || xx < 0 || xx >= p.W) return 0.f;
        const long long idx = (((long long)b * p.H + yy) * p.W + xx) * p.Cin + c;
        return p.a_f32 ? ((const float*)abase)[idx] : (float)((const __bf16*)abase)[idx];
    } else if (MODE == kDgrad) {
        if (m >= g.d_m || k >= g.kend) return 0.f;
        const int hw = g.d_hc * g.d_wc;
        const int b = m / hw, rem = m - b * hw;
        const int y = (rem / g.d_wc) * p.stride + g.d_ph, x = (rem % g.d_wc) * p.stride + g.d_pw;
        const int t = k / p.Cout, c = k - t * p.Cout, ir = t / g.d_ns, is = t - ir * g.d_ns;
        const int ty = y + p.pad - (g.d_r0 + ir * p.stride), tx = x + p.pad - (g.d_s0 + is * p.stride);
        const int yo = ty / p.stride, xo = tx / p.stride;
        if (ty < 0 || tx < 0 || yo >= p.Ho || xo >= p.Wo) return 0.f;
        return (float)((const __bf16*)abase)[(((long long)b * p.Ho + yo) * p.Wo + xo) * p.Cout + c];
    } else {
        const int mw = p.R * p.S * p.Cin;
        if (k >= g.kend) return 0.f;
        if (m == mw) return p.has_bias ? 1.f : 0.f;
        if (m > mw) return 0.f;
        const int hw = p.Ho * p.Wo;
        const int b = k / hw, rem = k - b * hw, yo = rem / p.Wo, xo = rem - yo * p.Wo;
        const int tap = m / p.Cin, c = m - tap * p.Cin, r = tap / p.S, s = tap - r * p.S;
        const int yy = yo * p.stride - p.pad + r, xx = xo * p.stride - p.pad + s;
        if (yy < 0 || yy >= p.H || xx < 0 || xx >= p.W) return 0.f;
        const long long idx = (((long long)b * p.H + yy) * p.W + xx) * p.Cin + c;
        return p.a_f32 ? ((const float*)abase)[idx] : (float)((const __bf16*)abase)[idx];
    }
}

template <int MODE>
__device__ __forceinline__ float fetch_b(const GemmParams& p, const Geo& g, const float* wbase, const __bf16* dybase, int k, int n)
{
    if (k >= g.kend || n >= p.N) return 0.f;
    if (MODE == kFwd) return wbase[(long long)k * p.N + n];
    if (MODE == kDgrad) {
        const int t = k / p.Cout, c = k - t * p.Cout, ir = t / g.d_ns, is = t - ir * g.d_ns;
        const int tap = (g.d_r0 + ir * p.stride) * p.S + g.d_s0 + is * p.stride;
        return wbase[((long long)tap * p.Cin + n) * p.Cout + c];
    }
    return (float)dybase[(long long)k * p.N + n];
}

template <int BM, int BN, int WM, int WN, int MODE>
__global__ __launch_bounds__(64 * WM * WN) void igemm_bf16_kernel(GemmParams p)
{
    constexpr int NT = 64 * WM * WN;
    constexpr int TM = BM / (WM * 32), TN = BN / (WN * 32);
    // k-contiguous slots: (row, group of 8 k): 4 per row.  pair slots: (pair of k, quad of rows): 16 * rows/4.
    constexpr int A_SLOTS = BM * 4, B_SLOTS = BN * 4;
    constexpr int NQA = (A_SLOTS + NT - 1) / NT, NQB = (B_SLOTS + NT - 1) / NT;
    static_assert(NT % BM == 0 || A_SLOTS <= NT, "");
    static_assert(NT % BN == 0 || B_SLOTS <= NT, "");
    static_assert(NT % 16 == 0, "");

    __shared__ __attribute__((aligned(16))) __bf16 sA[2][BM][LDP];
    __shared__ __attribute__((aligned(16))) __bf16 sB[2][BN][LDP];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int rep = p.order[blockIdx.z];
    const int tile_m = blockIdx.x / p.tiles_n, tile_n = blockIdx.x % p.tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int split = blockIdx.y;
    const int kbeg = (MODE == kDgrad) ? 0 : split * p.kchunk;

    const char* abase;
    if (p.cursor) {
        const long long first = (p.cursor[rep] * (long long)p.batch) % p.n_samples;
        abase = (const char*)p.a + ((long long)rep * p.n_samples + first) * p.sample_sz * 4;     // the data set is fp32
    } else {
        abase = (const char*)p.a + (long long)rep * p.a_rep * 4;
    }
    const float* wbase = p.w + (long long)rep * p.w_rep;
    const __bf16* dybase = (MODE == kWgrad) ? (const __bf16*)((const char*)p.dy + (long long)rep * p.dy_rep * 4) : nullptr;

    Geo g{};
    g.d_ns = p.S; g.d_hc = p.H; g.d_wc = p.W; g.d_m = p.M;
    g.kend = min(p.K, kbeg + p.kchunk);
    if (MODE == kDgrad) {
        g.d_ph = blockIdx.y / p.stride; g.d_pw = blockIdx.y % p.stride;
        g.d_hc = (p.H - g.d_ph + p.stride - 1) / p.stride; g.d_wc = (p.W - g.d_pw + p.stride - 1) / p.stride;
        g.d_r0 = (g.d_ph + p.pad) % p.stride; g.d_s0 = (g.d_pw + p.pad) % p.stride;
        const int nr = g.d_r0 < p.R ? (p.R - g.d_r0 + p.stride - 1) / p.stride : 0;
        g.d_ns = g.d_s0 < p.S ? (p.S - g.d_s0 + p.stride - 1) / p.stride : 0;
        g.d_m = p.B * g.d_hc * g.d_wc;
        g.kend = nr * g.d_ns * p.Cout;
        if (m0 >= g.d_m) return;
    }

    // vector paths need whole groups inside one tap / one row
    const bool vecA = !p.a_f32 && ((MODE == kFwd) ? (p.Cin % 8 == 0) : (MODE == kDgrad) ? (p.Cout % 8 == 0) : (p.Cin % 4 == 0));
    const bool vecB = (MODE == kFwd) ? (p.N % 4 == 0) : (MODE == kDgrad) ? (p.Cout % 8 == 0) : (p.N % 4 == 0);

    // loop-invariant row decomposition for the k-contiguous A loaders (one row per thread)
    int a_b = 0, a_y = 0, a_x = 0; bool a_ok = false;
    if (MODE != kWgrad) {
        const int m = m0 + (tid % BM);
        a_ok = m < ((MODE == kFwd) ? p.M : g.d_m);
        const int hw = (MODE == kFwd) ? p.Ho * p.Wo : g.d_hc * g.d_wc;
        const int ww = (MODE == kFwd) ? p.Wo : g.d_wc;
        a_b = m / hw;
        const int rem = m - a_b * hw;
        a_y = rem / ww; a_x = rem - a_y * ww;
        if (MODE == kDgrad) { a_y = a_y * p.stride + g.d_ph; a_x = a_x * p.stride + g.d_pw; }
    }

    // when the channel count is a multiple of the slab, a slab lies inside one filter tap and the tap arithmetic is
    // wave-uniform (done once per slab, not per slot)
    const bool slab_tap = (MODE == kFwd) ? (p.Cin % BK == 0) : (MODE == kDgrad) ? (p.Cout % BK == 0) : false;
    // weight-gradient A rows of this thread's pair slots: (tap, channel) of the first of 4 rows, fixed over the K loop
    int wa_r[NQA], wa_s[NQA], wa_c[NQA];
    if (MODE == kWgrad) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int m = m0 + ((tid + q * NT) / 16) * 4;
            const int tap = m / p.Cin;
            wa_c[q] = m - tap * p.Cin; wa_r[q] = tap / p.S; wa_s[q] = tap - wa_r[q] * p.S;
        }
    }

    u4 ra[NQA], rb[NQB];      // staged slot contents: 8 bf16 each

    auto load_tiles = [&](int k0) {
        int u_c0 = 0, u_dy = 0, u_dx = 0, u_tap = 0;      // slab-uniform tap (valid when slab_tap)
        if (slab_tap) {
            if (MODE == kFwd) {
                const int tap = k0 / p.Cin; u_c0 = k0 - tap * p.Cin;
                const int r = tap / p.S; u_dy = r - p.pad; u_dx = tap - r * p.S - p.pad;
            } else {
                const int t = k0 / p.Cout; u_c0 = k0 - t * p.Cout;
                const int ir = t / g.d_ns, is = t - ir * g.d_ns;
                u_dy = p.pad - (g.d_r0 + ir * p.stride); u_dx = p.pad - (g.d_s0 + is * p.stride);
                u_tap = (g.d_r0 + ir * p.stride) * p.S + g.d_s0 + is * p.stride;
            }
        }
        // ------------------------------------------------ A ------------------------------------------------
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int i = tid + q * NT;
            u4 v = {0u, 0u, 0u, 0u};
            if (i < A_SLOTS) {
                if (MODE != kWgrad) {
                    const int ml = i % BM, kq = i / BM, k = k0 + kq * 8;
                    if (vecA) {
                        if (a_ok && k < g.kend) {
                            if (MODE == kFwd) {
                                int c, dy, dx;
                                if (slab_tap) { c = u_c0 + kq * 8; dy = u_dy; dx = u_dx; }
                                else {
                                    const int tap = k / p.Cin, r = tap / p.S;
                                    c = k - tap * p.Cin; dy = r - p.pad; dx = tap - r * p.S - p.pad;
                                }
                                const int yy = a_y * p.stride + dy, xx = a_x * p.stride + dx;
                                if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W)
                                    v = *reinterpret_cast<const u4*>((const __bf16*)abase + (((long long)a_b * p.H + yy) * p.W + xx) * p.Cin + c);
                            } else {
                                int c, dy, dx;
                                if (slab_tap) { c = u_c0 + kq * 8; dy = u_dy; dx = u_dx; }
                                else {
                                    const int t = k / p.Cout, ir = t / g.d_ns, is = t - ir * g.d_ns;
                                    c = k - t * p.Cout; dy = p.pad - (g.d_r0 + ir * p.stride); dx = p.pad - (g.d_s0 + is * p.stride);
                                }
                                const int ty = a_y + dy, tx = a_x + dx;
                                const int yo = ty / p.stride, xo = tx / p.stride;
                                if (ty >= 0 && tx >= 0 && yo < p.Ho && xo < p.Wo)
                                    v = *reinterpret_cast<const u4*>((const __bf16*)abase + (((long long)a_b * p.Ho + yo) * p.Wo + xo) * p.Cout + c);
                            }
                        }
                    } else {
                        float f[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) f[j] = fetch_a<MODE>(p, g, abase, m0 + ml, k + j);
                        v = u4{pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7])};
                    }
                } else {
                    // pair slot: k pair kp, row quad rq; v[j] = (A[m+j][k], A[m+j][k+1])
                    const int kp = i % 16, rq = i / 16, k = k0 + 2 * kp, m = m0 + rq * 4;
                    const int mw = p.R * p.S * p.Cin;
                    if (vecA && m < mw) {
                        const int c = wa_c[q], r = wa_r[q], s = wa_s[q];
                        bf16x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
#pragma unroll
                        for (int h = 0; h < 2; ++h) {
                            const int kk = k + h;
                            if (kk < g.kend) {
                                int b, yo, xo;
                                if (p.hw_shift >= 0) {
                                    b = kk >> p.hw_shift;
                                    const int rem = kk & ((1 << p.hw_shift) - 1);
                                    yo = rem >> p.w_shift; xo = rem & ((1 << p.w_shift) - 1);
                                } else {
                                    const int hw = p.Ho * p.Wo;
                                    b = kk / hw;
                                    const int rem = kk - b * hw;
                                    yo = rem / p.Wo; xo = rem - yo * p.Wo;
                                }
                                const int yy = yo * p.stride - p.pad + r, xx = xo * p.stride - p.pad + s;
                                if (yy >= 0 && yy < p.H && xx >= 0 && xx < p.W) {
                                    const bf16x4 t = *reinterpret_cast<const bf16x4*>((const __bf16*)abase + (((long long)b * p.H + yy) * p.W + xx) * p.Cin + c);
                                    if (h == 0) lo = t; else hi = t;
                                }
                            }
                        }
                        v = u4{pack2b(lo[0], hi[0]), pack2b(lo[1], hi[1]), pack2b(lo[2], hi[2]), pack2b(lo[3], hi[3])};
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            v[j] = pack2(fetch_a<MODE>(p, g, abase, m + j, k), fetch_a<MODE>(p, g, abase, m + j, k + 1));
                    }
                }
            }
            ra[q] = v;
        }
        // ------------------------------------------------ B ------------------------------------------------
#pragma unroll
        for (int q = 0; q < NQB; ++q) {
            const int i = tid + q * NT;
            u4 v = {0u, 0u, 0u, 0u};
            if (i < B_SLOTS) {
                if (MODE == kDgrad) {
                    // k-contiguous: B[k = (tap, co)][n = ci] = W[tap][ci][co]
                    const int nl = i % BN, kq = i / BN, k = k0 + kq * 8, n = n0 + nl;
                    if (vecB) {
                        if (n < p.N && k < g.kend) {
                            int c, tap;
                            if (slab_tap) { c = u_c0 + kq * 8; tap = u_tap; }
                            else {
                                const int t = k / p.Cout, ir = t / g.d_ns, is = t - ir * g.d_ns;
                                c = k - t * p.Cout; tap = (g.d_r0 + ir * p.stride) * p.S + g.d_s0 + is * p.stride;
                            }
                            const float* src = wbase + ((long long)tap * p.Cin + n) * p.Cout + c;
                            const f4 x0 = *reinterpret_cast<const f4*>(src), x1 = *reinterpret_cast<const f4*>(src + 4);
                            v = u4{pack2(x0[0], x0[1]), pack2(x0[2], x0[3]), pack2(x1[0], x1[1]), pack2(x1[2], x1[3])};
                        }
                    } else {
                        float f[8];
#pragma unroll
                        for (int j = 0; j < 8; ++j) f[j] = fetch_b<MODE>(p, g, wbase, dybase, k + j, n);
                        v = u4{pack2(f[0], f[1]), pack2(f[2], f[3]), pack2(f[4], f[5]), pack2(f[6], f[7])};
                    }
                } else {
                    // pair slot: v[j] = (B[k][n+j], B[k+1][n+j])
                    const int kp = i % 16, rq = i / 16, k = k0 + 2 * kp, n = n0 + rq * 4;
                    if (vecB) {
                        if (n < p.N) {
                            if (MODE == kFwd) {
                                f4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};
                                if (k < g.kend) lo = *reinterpret_cast<const f4*>(wbase + (long long)k * p.N + n);
                                if (k + 1 < g.kend) hi = *reinterpret_cast<const f4*>(wbase + (long long)(k + 1) * p.N + n);
                                v = u4{pack2(lo[0], hi[0]), pack2(lo[1], hi[1]), pack2(lo[2], hi[2]), pack2(lo[3], hi[3])};
                            } else {
                                bf16x4 lo = {0, 0, 0, 0}, hi = {0, 0, 0, 0};
                                if (k < g.kend) lo = *reinterpret_cast<const bf16x4*>(dybase + (long long)k * p.N + n);
                                if (k + 1 < g.kend) hi = *reinterpret_cast<const bf16x4*>(dybase + (long long)(k + 1) * p.N + n);
                                v = u4{pack2b(lo[0], hi[0]), pack2b(lo[1], hi[1]), pack2b(lo[2], hi[2]), pack2b(lo[3], hi[3])};
                            }
                        }
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            v[j] = pack2(fetch_b<MODE>(p, g, wbase, dybase, k, n + j), fetch_b<MODE>(p, g, wbase, dybase, k + 1, n + j));
                    }
                }
            }
            rb[q] = v;
        }
    };

    auto store_tiles = [&](int buf) {
#pragma unroll
        for (int q = 0; q < NQA; ++q) {
            const int i = tid + q * NT;
            if (i < A_SLOTS) {
                if (MODE != kWgrad) {
                    *reinterpret_cast<u4*>(&sA[buf][i % BM][(i / BM) * 8]) = ra[q];
                } else {
                    const int kp = i % 16, rq = i / 16;
#pragma unroll
                    for (int j = 0; j < 4; ++j) *reinterpret_cast<unsigned*>(&sA[buf][rq * 4 + j][2 * kp]) = ra[q][j];
                }
            }
        }
#pragma unroll
        for (int q = 0; q < NQB; ++q) {
            const int i = tid + q * NT;
            if (i < B_SLOTS) {
                if (MODE == kDgrad) {
                    *reinterpret_cast<u4*>(&sB[buf][i % BN][(i / BN) * 8]) = rb[q];
                } else {
                    const int kp = i % 16, rq = i / 16;
#pragma unroll
                    for (int j = 0; j < 4; ++j) *reinterpret_cast<unsigned*>(&sB[buf][rq * 4 + j][2 * kp]) = rb[q][j];
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

    const int nslab = (g.kend - kbeg + BK - 1) / BK;
    if (nslab > 0) {
        load_tiles(kbeg);
        store_tiles(0);
    }
    __syncthreads();
    for (int t = 0; t < nslab; ++t) {
        const int buf = t & 1;
        if (t + 1 < nslab) load_tiles(kbeg + (t + 1) * BK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const int kof = ks * 16 + (lane >> 5) * 8;
            bf16x8 a[TM], b[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8*>(&sA[buf][(wm * TM + i) * 32 + (lane & 31)][kof]);
#pragma unroll
            for (int j = 0; j < TN; ++j) b[j] = *reinterpret_cast<const bf16x8*>(&sB[buf][(wn * TN + j) * 32 + (lane & 31)][kof]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (t + 1 < nslab) store_tiles(buf ^ 1);
        __syncthreads();
    }

    // ---------------- epilogue ----------------
    const float* bias = (MODE == kFwd && p.has_bias) ? (wbase + (long long)p.K * p.N) : nullptr;
    float* obase32 = nullptr; __bf16* obase16 = nullptr;
    if (MODE == kWgrad) {
        obase32 = (p.splits > 1) ? p.out + (long long)blockIdx.z * p.out_rep + (long long)split * p.out_split
                                 : p.out + (long long)rep * p.out_rep;
    } else {
        obase16 = (__bf16*)((char*)p.out + (long long)rep * p.out_rep * 4);
    }
    const __bf16* mask = (MODE == kDgrad && p.mask) ? (const __bf16*)((const char*)p.mask + (long long)rep * p.mask_rep * 4) : nullptr;
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
                if (m >= ((MODE == kDgrad) ? g.d_m : p.M)) continue;
                float r = acc[i][j][v];
                long long row = m;
                if (MODE == kDgrad && p.stride > 1) {
                    const int hw = g.d_hc * g.d_wc;
                    const int b = m / hw, rem = m - b * hw;
                    const int yy = rem / g.d_wc, xx = rem - yy * g.d_wc;
                    row = ((long long)b * p.H + yy * p.stride + g.d_ph) * p.W + xx * p.stride + g.d_pw;
                }
                const long long o = row * p.N + n;
                if (MODE == kWgrad) {
                    obase32[o] = r;
                } else if (MODE == kFwd) {
                    r += bv;
                    if (p.relu) r = fmaxf(r, 0.f);
                    obase16[o] = (__bf16)r;
                } else {
                    if (mask && !((float)mask[o] > 0.f)) r = 0.f;
                    if (p.accumulate) r += (float)obase16[o];
                    obase16[o] = (__bf16)r;
                }
            }
        }
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
        const int rows0 = p.B * ((p.H + p.stride - 1) / p.stride) * ((p.W + p.stride - 1) / p.stride);
        p.tiles_m = (rows0 + BM - 1) / BM;
    }
    const dim3 grid((unsigned)(p.tiles_m * p.tiles_n), gy, (unsigned)n_active), block(64 * WM * WN);
    switch (p.mode) {
    case kFwd: hipLaunchKernelGGL((igemm_bf16_kernel<BM, BN, WM, WN, kFwd>), grid, block, 0, s, p); break;
    case kDgrad: hipLaunchKernelGGL((igemm_bf16_kernel<BM, BN, WM, WN, kDgrad>), grid, block, 0, s, p); break;
    default: hipLaunchKernelGGL((igemm_bf16_kernel<BM, BN, WM, WN, kWgrad>), grid, block, 0, s, p); break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_bf16(const GemmParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1 || p.M < 1 || p.N < 1) return hipSuccess;
    const int bn = p.N > 64 ? 128 : (p.N > 32 ? 64 : 32);
    const long long blocks128 = (long long)((p.M + 127) / 128) * ((p.N + bn - 1) / bn) * p.splits * n_active;
    const bool tall = p.M >= 128 && blocks128 >= 256;
    if (bn == 128) return tall ? launch_tile<128, 128, 2, 2>(p, n_active, s) : launch_tile<64, 128, 1, 4>(p, n_active, s);
    if (bn == 64) return tall ? launch_tile<128, 64, 2, 2>(p, n_active, s) : launch_tile<64, 64, 2, 2>(p, n_active, s);
    return tall ? launch_tile<128, 32, 4, 1>(p, n_active, s) : launch_tile<32, 32, 1, 1>(p, n_active, s);
}

}  // namespace hadfl
