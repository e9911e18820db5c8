// bf16 configuration, first convolution of a network: its input is the fp32 data set (read through the replica's
// batch cursor) with very few channels, so the whole filter footprint K = R*S*Cin fits one MFMA contraction of 32.
// The general kernels spend their time gathering that operand through their scalar path; here
//   * forward: every lane gathers the 16 contraction values of its pixel straight into the MFMA operand (no LDS for
//     activations), the tiny weight matrix sits in LDS as bf16 [Cout][32], and the kernel is bound by its output write;
//   * weight gradient: the transposed operand [pixel][32] is built in LDS 64 pixels at a time next to the dY tile and
//     both are read with the transposing LDS read; column K of the operand is a constant 1, so row K of the result is
//     the bias gradient (the bias sits directly behind the weights in the parameter row).
// Arithmetic follows the bf16 configuration: inputs and weights rounded to bf16, fp32 accumulation, bias added in fp32.
#include "train_kernels.h"

namespace hadfl {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16 __attribute__((ext_vector_type(16)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef short s4v __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s4v lds_s4v;

constexpr int KP = 32;              // padded contraction length
constexpr int WP = 40;              // LDS pitch of a weight row in bf16 elements (80 bytes: conflict-free 16-byte reads)

// first sample row of the replica's current batch inside the data set
__device__ __forceinline__ const float* batch_base(const FirstConvParams& p, int rep)
{
    const long long first = (p.cursor[rep] * (long long)p.B) % p.n_samples;
    return p.x + ((long long)rep * p.n_samples + first) * (long long)(p.H * p.W * p.C);
}

// Footprint table, one entry per contraction index k < 32: (tap << 24) | (offset + 2^23), offset = element offset of
// (tap, channel) relative to the pixel's own first channel; entries beyond K have tap 31 (never valid).
__device__ __forceinline__ void build_table(const FirstConvParams& p, unsigned* tab)
{
    if (threadIdx.x < KP) {
        const int k = threadIdx.x;
        unsigned v = 31u << 24;
        if (k < p.K) {
            const int tap = k / p.C, ci = k - tap * p.C;
            const int r = tap / p.S, s = tap - r * p.S;
            const int off = ((r - p.pad) * p.W + (s - p.pad)) * p.C + ci;
            v = ((unsigned)tap << 24) | (unsigned)(off + (1 << 23));
        }
        tab[k] = v;
    }
}

struct Pixel { const float* ptr; unsigned taps; };    // first channel of the pixel; bit t set when tap t lies inside the image
__device__ __forceinline__ Pixel locate(const FirstConvParams& p, const float* xb, int m, bool live)
{
    Pixel q; q.ptr = xb; q.taps = 0;
    if (!live) return q;
    const int hw = p.H * p.W;
    const int b = m / hw, rem = m - b * hw, y = rem / p.W, x = rem - y * p.W;
    q.ptr = xb + (long long)m * p.C;
    unsigned rows = 0, cols = 0;                      // filter rows / columns that stay inside the image
    for (int r = 0; r < p.R; ++r) if (y + r - p.pad >= 0 && y + r - p.pad < p.H) rows |= 1u << r;
    for (int s = 0; s < p.S; ++s) if (x + s - p.pad >= 0 && x + s - p.pad < p.W) cols |= 1u << s;
    for (int r = 0; r < p.R; ++r) if ((rows >> r) & 1u) q.taps |= cols << (r * p.S);
    return q;
}
__device__ __forceinline__ float footprint(const Pixel& q, unsigned entry)
{
    return ((q.taps >> (entry >> 24)) & 1u) ? q.ptr[(int)(entry & 0xffffffu) - (1 << 23)] : 0.f;
}

// out[pixel][co] = sum_k footprint(pixel, k) * w[k][co] + bias[co]; 256 pixels per workgroup, 64 per wave
template <int TN>        // output channels = 32 * TN
__global__ __launch_bounds__(256) void conv_first_fwd_kernel(FirstConvParams p)
{
    __shared__ __attribute__((aligned(16))) __bf16 sW[32 * TN][WP];
    __shared__ unsigned tab[KP];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rep = p.order[blockIdx.y];
    const float* xb = batch_base(p, rep);
    const float* w = p.w + (long long)rep * p.w_rep;
    build_table(p, tab);
    for (int i = tid; i < 32 * TN * KP; i += 256) {
        const int n = i / KP, k = i - n * KP;
        sW[n][k] = (__bf16)(k < p.K ? w[(long long)k * p.N + n] : 0.f);
    }
    __syncthreads();

    const int m_wave = blockIdx.x * 256 + wave * 64;
    f16 acc[2][TN];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // all 32 gathers of the lane's two pixels are issued before the first product
    float raw[2][2][8];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int m = m_wave + i * 32 + (lane & 31);
        const Pixel q = locate(p, xb, m, m < p.M);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) raw[i][ks][e] = footprint(q, tab[ks * 16 + (lane >> 5) * 8 + e]);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 a;
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = (__bf16)raw[i][ks][e];
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bf16x8 bw = *reinterpret_cast<const bf16x8*>(&sW[j * 32 + (lane & 31)][ks * 16 + (lane >> 5) * 8]);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw, a, acc[i][j], 0, 0, 0);   // swapped: 4 channels per lane
            }
        }
    // A lane holds pixel (lane & 31) and channels 8*g + 4*(lane >> 5) + {0..3}: stored like that an instruction would
    // touch 32 rows with 16 bytes each.  Each wave passes its 32 x N block through LDS and writes whole rows instead.
    constexpr int SPB = 64 * TN + 16;                        // bytes per staged row
    __shared__ __attribute__((aligned(16))) char sOut[4][32 * SPB];
    char* const stage = sOut[wave];
    char* obase = (char*)p.out + (long long)rep * p.out_rep * 4;
    const float* bias = p.bias ? p.bias + (long long)rep * p.w_rep : nullptr;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = j * 32 + 8 * g + 4 * (lane >> 5);
                f4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]};
                if (bias) v += *reinterpret_cast<const f4*>(bias + n);
                if (p.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
                bf16x4 r;
#pragma unroll
                for (int e = 0; e < 4; ++e) r[e] = (__bf16)v[e];
                *reinterpret_cast<bf16x4*>(stage + (lane & 31) * SPB + n * 2) = r;
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int CPR = 4 * TN;                          // 16-byte chunks per row
        constexpr int RPI = 64 / CPR;                        // rows per instruction
#pragma unroll
        for (int t = 0; t < 32 / RPI; ++t) {
            const int row = lane / CPR + t * RPI, c = lane % CPR;
            const int m = m_wave + i * 32 + row;
            const u4 v = *reinterpret_cast<const u4*>(stage + row * SPB + c * 16);
            if (m < p.M) *reinterpret_cast<u4*>(obase + ((long long)m * p.N) * 2 + c * 16) = v;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
}

__device__ __forceinline__ bf16x8 lds_tr8(const char* base, unsigned off, unsigned pitch)
{
    const s4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v*)(base + off));
    const s4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s4v*)(base + off + 4 * pitch));
    typedef short s8v __attribute__((ext_vector_type(8)));
    const s8v v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, v);
}

// dW[k][co] (k < K), dbias[co] (row K) = sum over the pixels [split*kchunk, +kchunk) of footprint(pixel, k) * dy[pixel][co]
// Slabs of 128 pixels: thread t builds half the footprint (16 values) of pixel t / 2; wave w multiplies pixels 32w..32w+31.
template <int TN>
__global__ __launch_bounds__(256) void conv_first_wgrad_kernel(FirstConvParams p)
{
    constexpr int SL = 128;
    constexpr int PA = 192, PB = (32 * TN + 32) * 2;       // LDS pitches in bytes per pixel row (64 modulo 256: the rows a
                                                            // transposing read touches land in distinct banks)
    constexpr int RP = 32 * TN + 4;                         // floats per row of the reduction buffer
    constexpr int NQD = SL * 4 * TN / 256;                  // 16-byte dY chunks per thread
    static_assert(4 * 32 * RP * 4 <= SL * (PA + PB), "the reduction buffer reuses the operand tiles");
    __shared__ __attribute__((aligned(16))) char smem[SL * (PA + PB)];
    __shared__ unsigned tab[KP];
    char* const sA = smem;
    char* const sB = smem + SL * PA;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = blockIdx.y, rep = p.order[g], split = blockIdx.x;
    const float* xb = batch_base(p, rep);
    const char* dyb = (const char*)p.dy + (long long)rep * p.dy_rep * 4;
    const int kbeg = split * p.kchunk, kend = min(p.M, kbeg + p.kchunk);
    build_table(p, tab);
    __syncthreads();
    unsigned ent[16];
    const int pi = tid >> 1, kh = tid & 1;                  // operand builder: pixel pi of the slab, footprint values 16*kh..+15
#pragma unroll
    for (int e = 0; e < 16; ++e) ent[e] = tab[kh * 16 + e];
    const bool ones = p.bias && p.K / 16 == kh;             // this thread's half holds the bias column K
    const unsigned rd_lane = (unsigned)((lane >> 5) * 8 + ((lane & 15) >> 2));
    const unsigned col = (unsigned)((((lane >> 4) & 1) * 16 + (lane & 3) * 4) * 2);
    f16 acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;

    for (int k0 = kbeg; k0 < kend; k0 += SL) {
        const int m = k0 + pi;
        const bool live = m < kend;
        const Pixel q = locate(p, xb, m, live);
        float raw[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) raw[e] = footprint(q, ent[e]);
        if (ones && live) raw[p.K & 15] = 1.0f;                           // the bias column
        u4 dv[NQD];
#pragma unroll
        for (int c = 0; c < NQD; ++c) {
            const int i = tid + c * 256, r = i / (4 * TN), cc = i - r * (4 * TN);
            u4 v = {0u, 0u, 0u, 0u};
            if (k0 + r < kend) v = *reinterpret_cast<const u4*>(dyb + ((long long)(k0 + r) * p.N) * 2 + cc * 16);
            dv[c] = v;
        }
        __syncthreads();                                    // every wave is done reading the previous slab
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            bf16x8 a;
#pragma unroll
            for (int e = 0; e < 8; ++e) a[e] = (__bf16)raw[h * 8 + e];
            *reinterpret_cast<bf16x8*>(sA + pi * PA + (kh * 2 + h) * 16) = a;
        }
#pragma unroll
        for (int c = 0; c < NQD; ++c) {
            const int i = tid + c * 256, r = i / (4 * TN), cc = i - r * (4 * TN);
            *reinterpret_cast<u4*>(sB + r * PB + cc * 16) = dv[c];
        }
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const unsigned row = rd_lane + (unsigned)(wave * 32 + ks * 16);
            const bf16x8 a = lds_tr8(sA, row * PA + col, PA);
#pragma unroll
            for (int j = 0; j < TN; ++j) {
                const bf16x8 bv = lds_tr8(sB, row * PB + j * 64 + col, PB);
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bv, a, acc[j], 0, 0, 0);   // rows: footprint index, 4 channels per lane
            }
        }
    }
    // add the four waves' blocks in wave order, then store rows 0..K (K = bias row)
    __syncthreads();
    float (*sR)[32][RP] = reinterpret_cast<float (*)[32][RP]>(smem);
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f4 v = {acc[j][4 * q], acc[j][4 * q + 1], acc[j][4 * q + 2], acc[j][4 * q + 3]};
            *reinterpret_cast<f4*>(&sR[wave][lane & 31][j * 32 + 8 * q + 4 * (lane >> 5)]) = v;
        }
    __syncthreads();
    float* obase = (p.splits > 1) ? p.gout + (long long)g * p.gout_rep + (long long)split * p.gout_split
                                  : p.gout + (long long)rep * p.gout_rep;
    const int rows = p.K + (p.bias ? 1 : 0);
    for (int i = tid; i < rows * 8 * TN; i += 256) {
        const int m = i / (8 * TN), c4 = (i - m * (8 * TN)) * 4;
        const f4 s = ((*reinterpret_cast<const f4*>(&sR[0][m][c4]) + *reinterpret_cast<const f4*>(&sR[1][m][c4])) +
                      *reinterpret_cast<const f4*>(&sR[2][m][c4])) + *reinterpret_cast<const f4*>(&sR[3][m][c4]);
        *reinterpret_cast<f4*>(obase + (long long)m * p.N + c4) = s;
    }
}

}  // namespace

bool conv_first_supported(const FirstConvParams& p)
{
    return p.K + (p.bias ? 1 : 0) <= KP && (p.N == 32 || p.N == 64) && p.K == p.R * p.S * p.C;
}

hipError_t launch_conv_first_fwd(const FirstConvParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    if (!conv_first_supported(p)) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((p.M + 255) / 256), (unsigned)n_active), block(256);
    if (p.N == 32) hipLaunchKernelGGL(conv_first_fwd_kernel<1>, grid, block, 0, s, p);
    else hipLaunchKernelGGL(conv_first_fwd_kernel<2>, grid, block, 0, s, p);
    return hipGetLastError();
}

hipError_t launch_conv_first_wgrad(const FirstConvParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    if (!conv_first_supported(p) || p.splits < 1 || p.kchunk < 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)p.splits, (unsigned)n_active), block(256);
    if (p.N == 32) hipLaunchKernelGGL(conv_first_wgrad_kernel<1>, grid, block, 0, s, p);
    else hipLaunchKernelGGL(conv_first_wgrad_kernel<2>, grid, block, 0, s, p);
    return hipGetLastError();
}

}  // namespace hadfl
