// Memory-bound layers of the local-training path, grouped over the active replicas: ReLU, 2x2 max-pool,
// residual add, global average pool, batch normalisation (training mode), softmax cross-entropy and the fused
// SGD/momentum update.  All reductions run in a fixed order (no floating-point atomics): results are repeatable.
#include "train_kernels.h"

namespace hadfl {
namespace {

constexpr float kBwdStatCond = 16.f;    // largest |beta / gamma| for which y determines xhat well enough (bn_finalize_kernel)
constexpr float kBnEps = 1e-5f;
constexpr float kBnStatMomentum = 0.1f;

// Activation tensors are fp32 or bf16 (the bf16 configuration); offsets and per-replica strides are always counted
// in 4-byte units, so a bf16 tensor occupies the first half of its slot.
template <typename T> __device__ __forceinline__ T* tptr(const void* base, long long rep, long long rep_stride)
{
    return (T*)((char*)base + rep * rep_stride * 4);
}
__device__ __forceinline__ float ldf(const float* p, long long i) { return p[i]; }
__device__ __forceinline__ float ldf(const __bf16* p, long long i) { return (float)p[i]; }
__device__ __forceinline__ void stf(float* p, long long i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(__bf16* p, long long i, float v) { p[i] = (__bf16)v; }

__device__ __forceinline__ long long gtid() { return (long long)blockIdx.x * blockDim.x + threadIdx.x; }
__device__ __forceinline__ long long gstride() { return (long long)gridDim.x * blockDim.x; }

template <typename T>
__global__ __launch_bounds__(256) void relu_fwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* in = tptr<T>(p.in, rep, p.in_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    for (long long i = gtid(); i < p.count; i += gstride()) stf(out, i, fmaxf(ldf(in, i), 0.f));
}

template <typename T>
__global__ __launch_bounds__(256) void relu_bwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* x = tptr<T>(p.in, rep, p.in_rep);
    const T* dout = tptr<T>(p.in2, rep, p.in2_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        float g = ldf(x, i) > 0.f ? ldf(dout, i) : 0.f;
        if (mask && !(ldf(mask, i) > 0.f)) g = 0.f;
        stf(din, i, p.accumulate ? ldf(din, i) + g : g);
    }
}

// count = pooled elements; in is [B][H][W][C]
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* in = tptr<T>(p.in, rep, p.in_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    const int Ho = p.H / 2, Wo = p.W / 2;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const int c = (int)(i % p.C);
        long long t = i / p.C;
        const int xo = (int)(t % Wo); t /= Wo;
        const int yo = (int)(t % Ho);
        const int b = (int)(t / Ho);
        const long long q = (((long long)b * p.H + 2 * yo) * p.W + 2 * xo) * p.C + c;
        const long long rowp = (long long)p.W * p.C;
        stf(out, i, fmaxf(fmaxf(ldf(in, q), ldf(in, q + p.C)), fmaxf(ldf(in, q + rowp), ldf(in, q + rowp + p.C))));
    }
}

// the gradient goes to the first maximal element in (dy, dx) scan order; count = pooled elements
template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* x = tptr<T>(p.in, rep, p.in_rep);
    const T* dout = tptr<T>(p.in2, rep, p.in2_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const int Ho = p.H / 2, Wo = p.W / 2;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const int c = (int)(i % p.C);
        long long t = i / p.C;
        const int xo = (int)(t % Wo); t /= Wo;
        const int yo = (int)(t % Ho);
        const int b = (int)(t / Ho);
        const long long base = (((long long)b * p.H + 2 * yo) * p.W + 2 * xo) * p.C + c;
        const long long rowp = (long long)p.W * p.C;
        const long long off[4] = {0, p.C, rowp, rowp + p.C};
        float m = ldf(x, base); int arg = 0;
#pragma unroll
        for (int j = 1; j < 4; ++j) { const float v = ldf(x, base + off[j]); if (v > m) { m = v; arg = j; } }
        const float g = ldf(dout, i);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // with p.mask set, x is a fused ReLU output: the gradient passes only where it is positive
            const float v = (j == arg && (!p.mask || m > 0.f)) ? g : 0.f;
            const long long d = base + off[j];
            stf(din, d, p.accumulate ? ldf(din, d) + v : v);
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void add_fwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* a = tptr<T>(p.in, rep, p.in_rep);
    const T* b = tptr<T>(p.in2, rep, p.in2_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const float v = ldf(a, i) + ldf(b, i);
        stf(out, i, p.relu ? fmaxf(v, 0.f) : v);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void pass_grad_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* dout = tptr<T>(p.in, rep, p.in_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const float g = (!mask || ldf(mask, i) > 0.f) ? ldf(dout, i) : 0.f;
        stf(din, i, p.accumulate ? ldf(din, i) + g : g);
    }
}

// out[b][c] = mean over H*W; count = B*C
template <typename T>
__global__ __launch_bounds__(256) void gap_fwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* in = tptr<T>(p.in, rep, p.in_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    const int hw = p.H * p.W;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const int c = (int)(i % p.C);
        const long long b = i / p.C;
        float s = 0.f;
        for (int q = 0; q < hw; ++q) s += ldf(in, (b * hw + q) * p.C + c);
        stf(out, i, s / (float)hw);
    }
}

// din[b][q][c] (+)= dout[b][c] / (H*W); count = B*H*W*C
template <typename T>
__global__ __launch_bounds__(256) void gap_bwd_kernel(EwParams p)
{
    const int rep = p.order[blockIdx.y];
    const T* dout = tptr<T>(p.in, rep, p.in_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    const int hw = p.H * p.W;
    for (long long i = gtid(); i < p.count; i += gstride()) {
        const int c = (int)(i % p.C);
        const long long b = i / ((long long)hw * p.C);
        float g = ldf(dout, b * p.C + c) / (float)hw;
        if (mask && !(ldf(mask, i) > 0.f)) g = 0.f;
        stf(din, i, p.accumulate ? ldf(din, i) + g : g);
    }
}

// ------------------------------------------------------------------------------------------------------
// Batch normalisation over rows = B*H*W per channel.  Two reduction passes (sum, then squared deviation from
// the mean) keep the variance accurate in fp32; every pass writes per-chunk partial sums that the next kernel
// adds in chunk order.
// Block = 256 threads = 64 channel lanes x 4 row lanes; grid = (chunks * ceil(C/64), n_active).
// ------------------------------------------------------------------------------------------------------
template <int PASS, typename T>   // 0: sum x   1: sum (x-mean)^2   2 (backward): sum dy and sum dy*xhat
__global__ __launch_bounds__(256) void bn_reduce_kernel(BnParams p)
{
    __shared__ float red[2][4][64];
    const int g = blockIdx.y, rep = p.order[g];
    const int cgroups = (p.C + 63) / 64;
    const int chunk = blockIdx.x / cgroups, cg = blockIdx.x % cgroups;
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int c = cg * 64 + cl;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    float* part = p.partial + g * p.partial_rep;
    float mean = 0.f, istd = 0.f;
    if (PASS >= 1 && c < p.C) {
        if (PASS == 1) {
            float s = 0.f;
            for (int k = 0; k < p.chunks; ++k) s += part[((long long)k * 2 + 0) * p.C + c];
            mean = s / (float)p.rows;
        } else {
            const float* sv = p.saved + rep * p.saved_rep;
            mean = sv[c]; istd = sv[p.C + c];
        }
    }
    const int r0 = chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
    float s0 = 0.f, s1 = 0.f;
    if (c < p.C) {
        const T* dy = (PASS == 2) ? tptr<T>(p.dy, rep, p.dy_rep) : nullptr;
        for (int r = r0 + rl; r < r1; r += 4) {
            const float v = ldf(x, (long long)r * p.C + c);
            if (PASS == 0) s0 += v;
            else if (PASS == 1) { const float d = v - mean; s1 += d * d; }
            else { const float d = ldf(dy, (long long)r * p.C + c); s0 += d; s1 += d * ((v - mean) * istd); }
        }
    }
    red[0][rl][cl] = s0; red[1][rl][cl] = s1;
    __syncthreads();
    if (rl == 0 && c < p.C) {
        const float t0 = (red[0][0][cl] + red[0][1][cl]) + (red[0][2][cl] + red[0][3][cl]);
        const float t1 = (red[1][0][cl] + red[1][1][cl]) + (red[1][2][cl] + red[1][3][cl]);
        if (PASS == 0) part[((long long)chunk * 2 + 0) * p.C + c] = t0;
        else if (PASS == 1) part[((long long)chunk * 2 + 1) * p.C + c] = t1;
        else { part[((long long)chunk * 2 + 0) * p.C + c] = t0; part[((long long)chunk * 2 + 1) * p.C + c] = t1; }
    }
}

// y = gamma * (x - mean) * istd + beta; the blocks of chunk 0 also store mean / istd and update the running statistics
template <typename T>
__global__ __launch_bounds__(256) void bn_apply_fwd_kernel(BnParams p)
{
    const int g = blockIdx.y, rep = p.order[g];
    const int cgroups = (p.C + 63) / 64;
    const int chunk = blockIdx.x / cgroups, cg = blockIdx.x % cgroups;
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int c = cg * 64 + cl;
    if (c >= p.C) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    T* y = tptr<T>(p.y, rep, p.y_rep);
    const float* part = p.partial + g * p.partial_rep;
    float* row = p.params + rep * p.row_stride;
    float s = 0.f, q = 0.f;
    for (int k = 0; k < p.chunks; ++k) { s += part[((long long)k * 2 + 0) * p.C + c]; q += part[((long long)k * 2 + 1) * p.C + c]; }
    const float mean = s / (float)p.rows, var = q / (float)p.rows;
    const float istd = 1.0f / sqrtf(var + kBnEps);
    const float gamma = row[p.w_off + c], beta = row[p.w_off + p.C + c];
    if (chunk == 0 && rl == 0) {
        float* sv = p.saved + rep * p.saved_rep;
        sv[c] = mean; sv[p.C + c] = istd;
        const float unb = p.rows > 1 ? q / (float)(p.rows - 1) : var;
        float* rm = row + p.stat_off;
        rm[c] = (1.f - kBnStatMomentum) * rm[c] + kBnStatMomentum * mean;
        rm[p.C + c] = (1.f - kBnStatMomentum) * rm[p.C + c] + kBnStatMomentum * unb;
    }
    const int r0 = chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
    for (int r = r0 + rl; r < r1; r += 4) {
        const long long i = (long long)r * p.C + c;
        const float v = gamma * ((ldf(x, i) - mean) * istd) + beta;
        stf(y, i, p.relu ? fmaxf(v, 0.f) : v);
    }
}

// dx = gamma*istd*(dy - sum(dy)/n - xhat*sum(dy*xhat)/n); chunk-0 blocks write dgamma, dbeta
template <typename T>
__global__ __launch_bounds__(256) void bn_apply_bwd_kernel(BnParams p)
{
    const int g = blockIdx.y, rep = p.order[g];
    const int cgroups = (p.C + 63) / 64;
    const int chunk = blockIdx.x / cgroups, cg = blockIdx.x % cgroups;
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
    const int c = cg * 64 + cl;
    if (c >= p.C) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    const T* dy = tptr<T>(p.dy, rep, p.dy_rep);
    T* dx = tptr<T>(p.y, rep, p.y_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    const float* part = p.partial + g * p.partial_rep;
    const float* sv = p.saved + rep * p.saved_rep;
    float db = 0.f, dg = 0.f;
    for (int k = 0; k < p.chunks; ++k) { db += part[((long long)k * 2 + 0) * p.C + c]; dg += part[((long long)k * 2 + 1) * p.C + c]; }
    const float mean = sv[c], istd = sv[p.C + c];
    const float gamma = p.params[rep * p.row_stride + p.w_off + c];
    if (chunk == 0 && rl == 0) {
        float* gr = p.grads + rep * p.row_stride + p.w_off;
        gr[c] = dg; gr[p.C + c] = db;
    }
    const float inv_n = 1.0f / (float)p.rows, k1 = gamma * istd;
    const int r0 = chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
    for (int r = r0 + rl; r < r1; r += 4) {
        const long long i = (long long)r * p.C + c;
        const float xh = (ldf(x, i) - mean) * istd;
        float v = k1 * (ldf(dy, i) - db * inv_n - xh * dg * inv_n);
        if (mask && !(ldf(mask, i) > 0.f)) v = 0.f;
        stf(dx, i, p.accumulate ? ldf(dx, i) + v : v);
    }
}

// ------------------------------------------------------------------------------------------------------
// Vectorised batch-norm kernels (channel count a multiple of 16 bytes' worth of elements): a thread owns a vector of
// VEC consecutive channels (one 16-byte access per row) and strides over rows; a workgroup is CVB channel vectors x
// 256/CVB row lanes.  The forward statistics take ONE pass: sums of d = x - x0 and d^2 with x0 the tensor's first
// row (a shift close to the mean keeps  E[d^2] - E[d]^2  well conditioned), so forward is 2 passes and backward 2.
// ------------------------------------------------------------------------------------------------------
template <typename T> struct VecOf { static constexpr int n = 16 / (int)sizeof(T); };
typedef float f4v __attribute__((ext_vector_type(4)));
typedef __bf16 bf8v __attribute__((ext_vector_type(8)));

__device__ __forceinline__ void ldv(const float* p, long long i, float (&o)[4])
{
    const f4v v = *reinterpret_cast<const f4v*>(p + i);
    o[0] = v[0]; o[1] = v[1]; o[2] = v[2]; o[3] = v[3];
}
// (bf16 tensors of the large configuration are streamed once per pass and exceed the caches: non-temporal accesses
// measured 3 % faster over the BN kernels; the fp32 tensors of the smaller configurations measured slower with them)
__device__ __forceinline__ void ldv(const __bf16* p, long long i, float (&o)[8])
{
    const bf8v v = __builtin_nontemporal_load(reinterpret_cast<const bf8v*>(p + i));
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (float)v[e];
}
__device__ __forceinline__ void stv(float* p, long long i, const float (&o)[4])
{
    f4v v = {o[0], o[1], o[2], o[3]};
    *reinterpret_cast<f4v*>(p + i) = v;
}
__device__ __forceinline__ void stv(__bf16* p, long long i, const float (&o)[8])
{
    bf8v v;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] = (__bf16)o[e];
    __builtin_nontemporal_store(v, reinterpret_cast<bf8v*>(p + i));
}

// Element-wise kernels with 16-byte accesses for counts that are a multiple of VEC (same results as the scalar ones).
template <typename T>
__global__ __launch_bounds__(256) void add_fwd_vec_kernel(EwParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int rep = p.order[blockIdx.y];
    const T* a = tptr<T>(p.in, rep, p.in_rep);
    const T* b = tptr<T>(p.in2, rep, p.in2_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    const long long nvec = p.count / VEC;
    for (long long i = gtid(); i < nvec; i += gstride()) {
        float u[VEC], w[VEC];
        ldv(a, i * VEC, u); ldv(b, i * VEC, w);
#pragma unroll
        for (int e = 0; e < VEC; ++e) { const float v = u[e] + w[e]; u[e] = p.relu ? fmaxf(v, 0.f) : v; }
        stv(out, i * VEC, u);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void pass_grad_vec_kernel(EwParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int rep = p.order[blockIdx.y];
    const T* dout = tptr<T>(p.in, rep, p.in_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    const long long nvec = p.count / VEC;
    for (long long i = gtid(); i < nvec; i += gstride()) {
        float g[VEC];
        ldv(dout, i * VEC, g);
        if (mask) {
            float mk[VEC];
            ldv(mask, i * VEC, mk);
#pragma unroll
            for (int e = 0; e < VEC; ++e) if (!(mk[e] > 0.f)) g[e] = 0.f;
        }
        if (p.accumulate) {
            float old[VEC];
            ldv(din, i * VEC, old);
#pragma unroll
            for (int e = 0; e < VEC; ++e) g[e] = old[e] + g[e];
        }
        stv(din, i * VEC, g);
    }
}

// 2 x 2 max pooling, one thread per pooled pixel and group of VEC channels (16-byte accesses); count = pooled elements.
// Same results as the scalar kernels above, which stay for channel counts that are not a multiple of VEC.
template <typename T>
__global__ __launch_bounds__(256) void maxpool_fwd_vec_kernel(EwParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int rep = p.order[blockIdx.y];
    const T* in = tptr<T>(p.in, rep, p.in_rep);
    T* out = tptr<T>(p.out, rep, p.out_rep);
    const int Ho = p.H / 2, Wo = p.W / 2, CV = p.C / VEC;
    const long long nvec = p.count / VEC;
    const long long rowp = (long long)p.W * p.C;
    for (long long i = gtid(); i < nvec; i += gstride()) {
        const int cv = (int)(i % CV);
        long long t = i / CV;
        const int xo = (int)(t % Wo); t /= Wo;
        const int yo = (int)(t % Ho);
        const int b = (int)(t / Ho);
        const long long q = (((long long)b * p.H + 2 * yo) * p.W + 2 * xo) * p.C + cv * VEC;
        float a0[VEC], a1[VEC], a2[VEC], a3[VEC];
        ldv(in, q, a0); ldv(in, q + p.C, a1); ldv(in, q + rowp, a2); ldv(in, q + rowp + p.C, a3);
#pragma unroll
        for (int e = 0; e < VEC; ++e) a0[e] = fmaxf(fmaxf(a0[e], a1[e]), fmaxf(a2[e], a3[e]));
        stv(out, i * VEC, a0);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool_bwd_vec_kernel(EwParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int rep = p.order[blockIdx.y];
    const T* x = tptr<T>(p.in, rep, p.in_rep);
    const T* dout = tptr<T>(p.in2, rep, p.in2_rep);
    T* din = tptr<T>(p.out, rep, p.out_rep);
    const int Ho = p.H / 2, Wo = p.W / 2, CV = p.C / VEC;
    const long long nvec = p.count / VEC;
    const long long rowp = (long long)p.W * p.C;
    for (long long i = gtid(); i < nvec; i += gstride()) {
        const int cv = (int)(i % CV);
        long long t = i / CV;
        const int xo = (int)(t % Wo); t /= Wo;
        const int yo = (int)(t % Ho);
        const int b = (int)(t / Ho);
        const long long base = (((long long)b * p.H + 2 * yo) * p.W + 2 * xo) * p.C + cv * VEC;
        const long long off[4] = {0, p.C, rowp, rowp + p.C};
        float v[4][VEC], g[VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j) ldv(x, base + off[j], v[j]);
        ldv(dout, i * VEC, g);
        int arg[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            float m = v[0][e]; arg[e] = 0;
#pragma unroll
            for (int j = 1; j < 4; ++j) if (v[j][e] > m) { m = v[j][e]; arg[e] = j; }     // first maximum in scan order
            // with p.mask set, x is a fused ReLU output: the gradient passes only where it is positive
            if (p.mask && !(m > 0.f)) arg[e] = -1;
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float o[VEC];
            if (p.accumulate) ldv(din, base + off[j], o);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float w = (arg[e] == j) ? g[e] : 0.f;
                o[e] = p.accumulate ? o[e] + w : w;
            }
            stv(din, base + off[j], o);
        }
    }
}

struct BnGeo { int cvb, rl_count, cgroups, chunk, cv, rl, c; bool live; };
__device__ __forceinline__ BnGeo bn_geo(const BnParams& p, int vec)
{
    BnGeo g;
    const int CV = p.C / vec;
    g.cvb = p.cvb; g.rl_count = 256 / g.cvb;
    g.cgroups = (CV + g.cvb - 1) / g.cvb;
    g.chunk = blockIdx.x / g.cgroups;
    g.cv = (blockIdx.x % g.cgroups) * g.cvb + (threadIdx.x % g.cvb);
    g.rl = threadIdx.x / g.cvb;
    g.c = g.cv * vec;
    g.live = g.cv < CV;
    return g;
}

// MODE 0 (forward): partial[chunk][0] = sum(x - x0), [1] = sum((x - x0)^2)
// MODE 1 (backward): partial[chunk][0] = sum(dy), [1] = sum(dy * xhat)
template <int MODE, typename T>
__global__ __launch_bounds__(256) void bn_sums_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    __shared__ float red[256][2 * VEC + 1];
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    const T* dy = (MODE == 1) ? tptr<T>(p.dy, rep, p.dy_rep) : nullptr;
    float s0[VEC], s1[VEC], a[VEC], b[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { s0[e] = 0.f; s1[e] = 0.f; a[e] = 0.f; b[e] = 1.f; }
    if (g.live) {
        if (MODE == 0) ldv(x, g.c, a);                       // the shift: first row of the tensor
        else {
            const float* sv = p.saved + rep * p.saved_rep;
#pragma unroll
            for (int e = 0; e < VEC; ++e) { a[e] = sv[g.c + e]; b[e] = sv[p.C + g.c + e]; }
        }
        const int r0 = g.chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
#pragma unroll 4
        for (int r = r0 + g.rl; r < r1; r += g.rl_count) {
            float v[VEC];
            ldv(x, (long long)r * p.C + g.c, v);
            if (MODE == 0) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) { const float d = v[e] - a[e]; s0[e] += d; s1[e] += d * d; }
            } else {
                float d[VEC];
                ldv(dy, (long long)r * p.C + g.c, d);
#pragma unroll
                for (int e = 0; e < VEC; ++e) { s0[e] += d[e]; s1[e] += d[e] * ((v[e] - a[e]) * b[e]); }
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) { red[threadIdx.x][e] = s0[e]; red[threadIdx.x][VEC + e] = s1[e]; }
    __syncthreads();
    for (int w = g.rl_count / 2; w > 0; w >>= 1) {           // fixed-order tree over the row lanes
        if (g.rl < w) {
#pragma unroll
            for (int e = 0; e < 2 * VEC; ++e) red[threadIdx.x][e] += red[threadIdx.x + w * g.cvb][e];
        }
        __syncthreads();
    }
    if (g.rl == 0 && g.live) {
        float* part = p.partial + gi * p.partial_rep + (long long)g.chunk * 2 * p.C;
#pragma unroll
        for (int e = 0; e < VEC; ++e) { part[g.c + e] = red[threadIdx.x][e]; part[p.C + g.c + e] = red[threadIdx.x][VEC + e]; }
    }
}

struct PoolWin { long long q[4]; long long o; };
__device__ __forceinline__ PoolWin pool_window(const BnParams& p, int w, int c)
{
    const int Wo = p.W / 2, Ho = p.H / 2;
    const int xo = w % Wo; int t = w / Wo;
    const int yo = t % Ho, b = t / Ho;
    PoolWin r;
    r.q[0] = (((long long)b * p.H + 2 * yo) * p.W + 2 * xo) * p.C + c;
    r.q[1] = r.q[0] + p.C; r.q[2] = r.q[0] + (long long)p.W * p.C; r.q[3] = r.q[2] + p.C;
    r.o = (long long)w * p.C + c;
    return r;
}

// A workgroup takes 32 channels; eight threads per channel add the per-chunk partial sums (chunks k, k+8, ..) and a
// fixed-order tree over the eight joins them.
// Scale and shift of the normalisation and the stored output of one element.  The kernels of a batch norm with a
// folded max-pool do not keep the full-resolution output: the backward ones form a window's four outputs again from x.
// Both directions go through these two functions -- explicit fused multiply-adds, the rounding of the stored type --
// so the values compared for the window's maximum are bit for bit the ones the forward pass took the maximum of.
__device__ __forceinline__ void bn_scale_shift(float mean, float istd, float gamma, float beta, float& sc, float& sh)
{
    sc = gamma * istd;
    sh = __builtin_fmaf(-mean, sc, beta);
}
__device__ __forceinline__ float bn_value(float x, float sc, float sh, bool relu)
{
    const float t = __builtin_fmaf(x, sc, sh);
    return relu ? fmaxf(t, 0.f) : t;
}
template <typename T> __device__ __forceinline__ float bn_stored_value(float x, float sc, float sh, bool relu)
{
    return (float)(T)bn_value(x, sc, sh, relu);
}

// MODE 0: mean and 1/sqrt(var+eps) -> saved, running statistics updated.  x0 is the shift used by the sums pass.
// MODE 1: totals of dy and dy*xhat -> gradient of beta and gamma, and into chunk 0 of the partial buffer.
template <int MODE, typename T>
__global__ __launch_bounds__(256) void bn_finalize_kernel(BnParams p)
{
    __shared__ float red[8][32][2];
    const int gi = blockIdx.y, rep = p.order[gi];
    const int cl = threadIdx.x & 31, kl = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + cl;
    const bool live = c < p.C;
    float* part = p.partial + gi * p.partial_rep;
    const int nk = ((MODE == 0 && p.stats_done) || (MODE == 1 && p.bwd_stats_done)) ? p.stat_entries : p.chunks;
    float s = 0.f, q = 0.f;
    // Backward sums left by the data gradient above are s = sum g and q = sum g * y, y = gamma * xhat + beta the stored
    // (bf16) output, so that  sum g * xhat = (q - beta * s) / gamma.  The bf16 rounding of y enters xhat multiplied by
    // |y / gamma| <= |xhat| + |beta / gamma|: harmless while |beta| <= kBwdStatCond * |gamma| (every trained net's
    // case; the rounding errors of the terms are independent and average out in the sum), useless when gamma is zero
    // or tiny beside beta.  Channels outside that range are summed again from x and the gradient, exactly as the sums
    // kernels do, by the whole workgroup, one channel after the other (slow, and rare).
    float gamma = 1.f, beta = 0.f;
    bool direct = false;
    if (MODE == 1) {
        __shared__ int s_direct[32];
        __shared__ float s_sum[32][2];
        __shared__ float s_red[256][2];
        if (p.bwd_stats_done && live) {
            const float* row = p.params + rep * p.row_stride + p.w_off;
            gamma = row[c]; beta = row[p.C + c];
            direct = gamma == 0.f || !(fabsf(beta) <= kBwdStatCond * fabsf(gamma));
        }
        if (kl == 0) s_direct[cl] = direct ? 1 : 0;
        __syncthreads();
        for (int j = 0; j < 32; ++j) {
            if (!s_direct[j]) continue;                       // uniform over the workgroup
            const int cj = blockIdx.x * 32 + j;
            const T* x = tptr<T>(p.x, rep, p.x_rep);
            const float* sv = p.saved + rep * p.saved_rep;
            const float mean = sv[cj], istd = sv[p.C + cj];
            float ts = 0.f, tq = 0.f;
            if (!p.pool) {
                const T* dy = tptr<T>(p.dy, rep, p.dy_rep);
                for (int r = threadIdx.x; r < p.rows; r += 256) {
                    const float d = ldf(dy, (long long)r * p.C + cj);
                    ts += d; tq += d * ((ldf(x, (long long)r * p.C + cj) - mean) * istd);
                }
            } else {
                const T* pg = tptr<T>(p.pool_g, rep, p.pool_g_rep);
                const float* row = p.params + rep * p.row_stride + p.w_off;
                float sc, sh;
                bn_scale_shift(mean, istd, row[cj], row[p.C + cj], sc, sh);
                for (int w = threadIdx.x; w < p.rows / 4; w += 256) {
                    const PoolWin pw = pool_window(p, w, cj);
                    float xw[4];
                    for (int t = 0; t < 4; ++t) xw[t] = ldf(x, pw.q[t]);
                    float m = bn_stored_value<T>(xw[0], sc, sh, p.relu != 0), xs = xw[0];
                    for (int t = 1; t < 4; ++t) {             // first maximum of the window's (recomputed) outputs
                        const float v = bn_stored_value<T>(xw[t], sc, sh, p.relu != 0);
                        if (v > m) { m = v; xs = xw[t]; }
                    }
                    if (p.relu && !(m > 0.f)) continue;       // the fused ReLU passes nothing there
                    const float d = ldf(pg, pw.o);
                    ts += d; tq += d * ((xs - mean) * istd);
                }
            }
            s_red[threadIdx.x][0] = ts; s_red[threadIdx.x][1] = tq;
            __syncthreads();
            for (int w = 128; w > 0; w >>= 1) {               // fixed-order tree
                if ((int)threadIdx.x < w) { s_red[threadIdx.x][0] += s_red[threadIdx.x + w][0]; s_red[threadIdx.x][1] += s_red[threadIdx.x + w][1]; }
                __syncthreads();
            }
            if (threadIdx.x == 0) { s_sum[j][0] = s_red[0][0]; s_sum[j][1] = s_red[0][1]; }
            __syncthreads();
        }
        if (direct && kl == 0) { s = s_sum[cl][0]; q = s_sum[cl][1]; }
    }
    if (live && !direct) {
        // (up to a thousand entries per lane after a convolution with small tiles: keep many loads in flight; the
        // additions stay in ascending order)
#pragma unroll 16
        for (int k = kl; k < nk; k += 8) { s += part[(long long)k * 2 * p.C + c]; q += part[(long long)k * 2 * p.C + p.C + c]; }
    }
    red[kl][cl][0] = s; red[kl][cl][1] = q;
    __syncthreads();
    for (int w = 4; w > 0; w >>= 1) {
        if (kl < w) { red[kl][cl][0] += red[kl + w][cl][0]; red[kl][cl][1] += red[kl + w][cl][1]; }
        __syncthreads();
    }
    if (kl != 0 || !live) return;
    s = red[0][cl][0]; q = red[0][cl][1];
    if (MODE == 0) {
        const float n = (float)p.rows;
        // the shift the sums were taken with: the producing convolution's bias, or the tensor's first row
        const float x0 = p.stats_done ? (p.stat_shift ? p.stat_shift[rep * p.stat_shift_rep + c] : 0.f)
                                      : ldf(tptr<T>(p.x, rep, p.x_rep), c);
        const float md = s / n;                               // mean of the shifted values
        const float cen = fmaxf(q - s * md, 0.f);             // sum of squared deviations from the mean
        const float mean = x0 + md, var = cen / n;
        float* sv = p.saved + rep * p.saved_rep;
        sv[c] = mean; sv[p.C + c] = 1.0f / sqrtf(var + kBnEps);
        const float unb = p.rows > 1 ? cen / (n - 1.f) : var;
        float* rm = p.params + rep * p.row_stride + p.stat_off;
        rm[c] = (1.f - kBnStatMomentum) * rm[c] + kBnStatMomentum * mean;
        rm[p.C + c] = (1.f - kBnStatMomentum) * rm[p.C + c] + kBnStatMomentum * unb;
    } else {
        if (p.bwd_stats_done && !direct) q = (q - beta * s) / gamma;
        float* gr = p.grads + rep * p.row_stride + p.w_off;
        gr[c] = q; gr[p.C + c] = s;
        part[c] = s; part[p.C + c] = q;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_apply_fwd_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    if (!g.live) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    T* y = tptr<T>(p.y, rep, p.y_rep);
    const float* row = p.params + rep * p.row_stride;
    float sc[VEC], sh[VEC];
    const float* sv = p.saved + rep * p.saved_rep;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int c = g.c + e;
        bn_scale_shift(sv[c], sv[p.C + c], row[p.w_off + c], row[p.w_off + p.C + c], sc[e], sh[e]);
    }
    const int r0 = g.chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
#pragma unroll 4
    for (int r = r0 + g.rl; r < r1; r += g.rl_count) {
        float v[VEC];
        const long long i = (long long)r * p.C + g.c;
        ldv(x, i, v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) v[e] = bn_value(v[e], sc[e], sh[e], p.relu != 0);
        stv(y, i, v);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_apply_bwd_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    if (!g.live) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    const T* dy = tptr<T>(p.dy, rep, p.dy_rep);
    T* dx = tptr<T>(p.y, rep, p.y_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    const float* part = p.partial + gi * p.partial_rep;
    const float* sv = p.saved + rep * p.saved_rep;
    const float inv_n = 1.0f / (float)p.rows;
    float mean[VEC], istd[VEC], k1[VEC], kb[VEC], kg[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int c = g.c + e;
        const float db = part[c], dg = part[p.C + c];       // totals left in chunk 0 by bn_finalize_kernel<1>
        mean[e] = sv[c]; istd[e] = sv[p.C + c];
        k1[e] = p.params[rep * p.row_stride + p.w_off + c] * istd[e];
        kb[e] = db * inv_n; kg[e] = dg * inv_n;
    }
    const int r0 = g.chunk * p.chunk_rows, r1 = min(p.rows, r0 + p.chunk_rows);
#pragma unroll 4
    for (int r = r0 + g.rl; r < r1; r += g.rl_count) {
        const long long i = (long long)r * p.C + g.c;
        float v[VEC], d[VEC], o[VEC];
        ldv(x, i, v); ldv(dy, i, d);
#pragma unroll
        for (int e = 0; e < VEC; ++e) o[e] = k1[e] * (d[e] - kb[e] - ((v[e] - mean[e]) * istd[e]) * kg[e]);
        if (mask) {
            float mk[VEC];
            ldv(mask, i, mk);
#pragma unroll
            for (int e = 0; e < VEC; ++e) if (!(mk[e] > 0.f)) o[e] = 0.f;
        }
        if (p.accumulate) {
            float old[VEC];
            ldv(dx, i, old);
#pragma unroll
            for (int e = 0; e < VEC; ++e) o[e] += old[e];
        }
        stv(dx, i, o);
    }
}

// ------------------------------------------------------------------------------------------------------
// Batch norm whose (ReLU'd) output feeds a 2x2/stride-2 max-pool only: the pool is folded into the BN kernels.
// A thread walks 2x2 windows instead of single rows.  Forward: it normalises the four pixels, stores them and their
// maximum (one pass less over the full-resolution tensor than a separate pool).  Backward: the gradient of a pixel
// is the pooled gradient where the pixel is the window's first maximum in scan order and is positive, else zero; it
// is formed on the fly from the stored output and the pooled gradient, so the full-resolution gradient tensor is
// neither written nor read (two passes less).  Window w of chunk c: [c * chunk_windows, (c + 1) * chunk_windows).
// ------------------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void bn_apply_fwd_pool_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    if (!g.live) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    T* po = tptr<T>(p.pool_out, rep, p.pool_out_rep);
    const float* row = p.params + rep * p.row_stride;
    float sc[VEC], sh[VEC];
    const float* sv = p.saved + rep * p.saved_rep;
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int c = g.c + e;
        bn_scale_shift(sv[c], sv[p.C + c], row[p.w_off + c], row[p.w_off + p.C + c], sc[e], sh[e]);
    }
    const int windows = p.rows / 4, cw = (windows + p.chunks - 1) / p.chunks;
    const int w0 = g.chunk * cw, w1 = min(windows, w0 + cw);
#pragma unroll 2
    for (int w = w0 + g.rl; w < w1; w += g.rl_count) {
        const PoolWin pw = pool_window(p, w, g.c);
        float v[4][VEC], m[VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j) ldv(x, pw.q[j], v[j]);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) v[j][e] = bn_value(v[j][e], sc[e], sh[e], p.relu != 0);
        }                                                     // (the four outputs themselves are not stored)
#pragma unroll
        for (int e = 0; e < VEC; ++e) m[e] = fmaxf(fmaxf(v[0][e], v[1][e]), fmaxf(v[2][e], v[3][e]));
        stv(po, pw.o, m);
    }
}

// which of the window's four pixels receives the pooled gradient (per channel), or -1
template <int VEC>
__device__ __forceinline__ void pool_argmax(const float (&yv)[4][VEC], bool relu, int (&arg)[VEC])
{
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        float m = yv[0][e]; arg[e] = 0;
#pragma unroll
        for (int j = 1; j < 4; ++j) if (yv[j][e] > m) { m = yv[j][e]; arg[e] = j; }     // first maximum in scan order
        if (relu && !(m > 0.f)) arg[e] = -1;                                             // the fused ReLU passes nothing there
    }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_sums_pool_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    __shared__ float red[256][2 * VEC + 1];
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    const T* pg = tptr<T>(p.pool_g, rep, p.pool_g_rep);
    float s0[VEC], s1[VEC], a[VEC], b[VEC], sc[VEC], sh[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) { s0[e] = 0.f; s1[e] = 0.f; a[e] = 0.f; b[e] = 1.f; sc[e] = 0.f; sh[e] = 0.f; }
    if (g.live) {
        const float* sv = p.saved + rep * p.saved_rep;
        const float* row = p.params + rep * p.row_stride + p.w_off;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            a[e] = sv[g.c + e]; b[e] = sv[p.C + g.c + e];
            bn_scale_shift(a[e], b[e], row[g.c + e], row[p.C + g.c + e], sc[e], sh[e]);
        }
        const int windows = p.rows / 4, cw = (windows + p.chunks - 1) / p.chunks;
        const int w0 = g.chunk * cw, w1 = min(windows, w0 + cw);
#pragma unroll 2
        for (int w = w0 + g.rl; w < w1; w += g.rl_count) {
            const PoolWin pw = pool_window(p, w, g.c);
            float yv[4][VEC], xv[4][VEC], gv[VEC];
            int arg[VEC];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ldv(x, pw.q[j], xv[j]);
#pragma unroll
                for (int e = 0; e < VEC; ++e) yv[j][e] = bn_stored_value<T>(xv[j][e], sc[e], sh[e], p.relu != 0);
            }
            ldv(pg, pw.o, gv);
            pool_argmax<VEC>(yv, p.relu != 0, arg);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                float xs = xv[0][e];
#pragma unroll
                for (int j = 1; j < 4; ++j) xs = arg[e] == j ? xv[j][e] : xs;
                const float d = arg[e] >= 0 ? gv[e] : 0.f;
                s0[e] += d; s1[e] += d * ((xs - a[e]) * b[e]);
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) { red[threadIdx.x][e] = s0[e]; red[threadIdx.x][VEC + e] = s1[e]; }
    __syncthreads();
    for (int w = g.rl_count / 2; w > 0; w >>= 1) {           // fixed-order tree over the row lanes
        if (g.rl < w) {
#pragma unroll
            for (int e = 0; e < 2 * VEC; ++e) red[threadIdx.x][e] += red[threadIdx.x + w * g.cvb][e];
        }
        __syncthreads();
    }
    if (g.rl == 0 && g.live) {
        float* part = p.partial + gi * p.partial_rep + (long long)g.chunk * 2 * p.C;
#pragma unroll
        for (int e = 0; e < VEC; ++e) { part[g.c + e] = red[threadIdx.x][e]; part[p.C + g.c + e] = red[threadIdx.x][VEC + e]; }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void bn_apply_bwd_pool_vec_kernel(BnParams p)
{
    constexpr int VEC = VecOf<T>::n;
    const int gi = blockIdx.y, rep = p.order[gi];
    const BnGeo g = bn_geo(p, VEC);
    if (!g.live) return;
    const T* x = tptr<T>(p.x, rep, p.x_rep);
    const T* pg = tptr<T>(p.pool_g, rep, p.pool_g_rep);
    T* dx = tptr<T>(p.y, rep, p.y_rep);
    const T* mask = p.mask ? tptr<T>(p.mask, rep, p.mask_rep) : nullptr;
    const float* part = p.partial + gi * p.partial_rep;
    const float* sv = p.saved + rep * p.saved_rep;
    const float inv_n = 1.0f / (float)p.rows;
    float mean[VEC], istd[VEC], k1[VEC], kb[VEC], kg[VEC], sc[VEC], sh[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int c = g.c + e;
        const float db = part[c], dg = part[p.C + c];       // totals left in chunk 0 by bn_finalize_kernel<1>
        const float* row = p.params + rep * p.row_stride + p.w_off;
        mean[e] = sv[c]; istd[e] = sv[p.C + c];
        k1[e] = row[c] * istd[e];
        kb[e] = db * inv_n; kg[e] = dg * inv_n;
        bn_scale_shift(mean[e], istd[e], row[c], row[p.C + c], sc[e], sh[e]);
    }
    const int windows = p.rows / 4, cw = (windows + p.chunks - 1) / p.chunks;
    const int w0 = g.chunk * cw, w1 = min(windows, w0 + cw);
#pragma unroll 2
    for (int w = w0 + g.rl; w < w1; w += g.rl_count) {
        const PoolWin pw = pool_window(p, w, g.c);
        float yv[4][VEC], xv[4][VEC], gv[VEC];
        int arg[VEC];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ldv(x, pw.q[j], xv[j]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) yv[j][e] = bn_stored_value<T>(xv[j][e], sc[e], sh[e], p.relu != 0);
        }
        ldv(pg, pw.o, gv);
        pool_argmax<VEC>(yv, p.relu != 0, arg);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float o[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float d = arg[e] == j ? gv[e] : 0.f;
                o[e] = k1[e] * (d - kb[e] - ((xv[j][e] - mean[e]) * istd[e]) * kg[e]);
            }
            if (mask) {
                float mk[VEC];
                ldv(mask, pw.q[j], mk);
#pragma unroll
                for (int e = 0; e < VEC; ++e) if (!(mk[e] > 0.f)) o[e] = 0.f;
            }
            if (p.accumulate) {
                float old[VEC];
                ldv(dx, pw.q[j], old);
#pragma unroll
                for (int e = 0; e < VEC; ++e) o[e] += old[e];
            }
            stv(dx, pw.q[j], o);
        }
    }
}

// One workgroup per replica, one thread per sample: softmax, loss, d(loss)/d(logits); loss summed by an LDS tree.
template <typename T>
__global__ __launch_bounds__(1024) void softmax_ce_kernel(LossParams p)
{
    __shared__ float red[1024];
    const int rep = p.order[blockIdx.x];
    const int b = threadIdx.x;
    float li = 0.f;
    if (b < p.batch) {
        const long long first = (p.cursor[rep] * (long long)p.batch) % p.n_samples;
        const int label = p.y[(long long)rep * p.n_samples + first + b];
        const T* z = tptr<T>(p.logits, rep, p.logits_rep) + (long long)b * p.n_classes;
        T* dz = tptr<T>(p.dlogits, rep, p.dlogits_rep) + (long long)b * p.n_classes;
        float m = ldf(z, 0);
        for (int j = 1; j < p.n_classes; ++j) m = fmaxf(m, ldf(z, j));
        float s = 0.f;
        for (int j = 0; j < p.n_classes; ++j) s += expf(ldf(z, j) - m);
        li = (logf(s) + m - ldf(z, label)) / (float)p.batch;
        const float inv = 1.0f / s;
        for (int j = 0; j < p.n_classes; ++j)
            stf(dz, j, (expf(ldf(z, j) - m) * inv - (j == label ? 1.f : 0.f)) / (float)p.batch);
    }
    red[b] = li;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if (b < w) red[b] += red[b + w];
        __syncthreads();
    }
    if (b == 0) p.loss[rep] = red[0];
}

typedef float f4 __attribute__((ext_vector_type(4)));

// buf = momentum*buf + g; w = w - lr*buf (local-update equation; momentum 0 is the paper's form).
__global__ __launch_bounds__(256) void sgd_kernel(SgdParams p)
{
    const int rep = p.order[blockIdx.y];
    float* const w = p.w + rep * p.row_stride;
    const float* const g = p.g + rep * p.row_stride;
    float* const buf = p.buf ? p.buf + rep * p.row_stride : nullptr;
    long long n4 = 0;
    for (int k = 0; k < p.n_seg; ++k) n4 += p.count[k] / 4;
    for (long long i = gtid(); i < n4; i += gstride()) {
        long long j = i; int k = 0;
        while (j >= p.count[k] / 4) { j -= p.count[k] / 4; ++k; }       // piece k, vector j of it
        const long long o = p.first[k] + 4 * j;
        f4 d = *reinterpret_cast<const f4*>(g + o);
        if (buf) { d = *reinterpret_cast<const f4*>(buf + o) * p.momentum + d; *reinterpret_cast<f4*>(buf + o) = d; }
        *reinterpret_cast<f4*>(w + o) = *reinterpret_cast<const f4*>(w + o) - d * p.lr;
    }
    if (p.bump && blockIdx.x == 0 && threadIdx.x == 0) { p.cursor[rep] += 1; p.versions[rep] += 1; }
}

// Narrow dense layer (the classifier: out <= 16): one workgroup per sample row; threads stride over the input
// features, keep `out` partial sums each and combine them with a fixed butterfly and a fixed LDS order.  Too small
// for the matrix cores.
template <int NMAX, typename T>
__global__ __launch_bounds__(256) void dense_small_fwd_kernel(DenseSmallParams p)
{
    __shared__ float red[4][NMAX];
    const int rep = p.order[blockIdx.y];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int m = blockIdx.x;
    const T* x = tptr<T>(p.x, rep, p.x_rep) + (long long)m * p.K;
    const float* w = p.w + rep * p.w_rep;
    constexpr bool kRoundW = sizeof(T) == 2;      // bf16 configuration: weights take part rounded to bf16
    float acc[NMAX];
#pragma unroll
    for (int n = 0; n < NMAX; ++n) acc[n] = 0.f;
    for (int k = threadIdx.x; k < p.K; k += 256) {
        const float xv = ldf(x, k);
        const float* wr = w + (long long)k * p.N;
#pragma unroll
        for (int n = 0; n < NMAX; ++n) if (n < p.N) acc[n] += xv * (kRoundW ? (float)(__bf16)wr[n] : wr[n]);
    }
#pragma unroll
    for (int n = 0; n < NMAX; ++n) {
        float v = acc[n];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
        if (lane == 0) red[wave][n] = v;
    }
    __syncthreads();
    if (threadIdx.x < p.N) {
        const int n = threadIdx.x;
        T* o = tptr<T>(p.out, rep, p.out_rep) + (long long)m * p.N;
        stf(o, n, ((red[0][n] + red[1][n]) + (red[2][n] + red[3][n])) + (p.has_bias ? w[(long long)p.K * p.N + n] : 0.f));
    }
}

dim3 ew_grid(long long count, int n_active)
{
    long long b = (count + 255) / 256;
    if (b > 2048) b = 2048;
    if (b < 1) b = 1;
    return dim3((unsigned)b, (unsigned)n_active);
}

}  // namespace

#define HADFL_EW_LAUNCH(fn, kern) \
    hipError_t fn(const EwParams& p, int n_active, hipStream_t s) { \
        if (n_active < 1 || p.count < 1) return hipSuccess; \
        if (p.bf16) hipLaunchKernelGGL(kern<__bf16>, ew_grid(p.count, n_active), dim3(256), 0, s, p); \
        else hipLaunchKernelGGL(kern<float>, ew_grid(p.count, n_active), dim3(256), 0, s, p); \
        return hipGetLastError(); }
HADFL_EW_LAUNCH(launch_relu_fwd, relu_fwd_kernel)
HADFL_EW_LAUNCH(launch_relu_bwd, relu_bwd_kernel)
HADFL_EW_LAUNCH(launch_gap_fwd, gap_fwd_kernel)
HADFL_EW_LAUNCH(launch_gap_bwd, gap_bwd_kernel)
#undef HADFL_EW_LAUNCH

#define HADFL_EW_VEC_LAUNCH(fn, vkern, kern) \
    hipError_t fn(const EwParams& p, int n_active, hipStream_t s) { \
        if (n_active < 1 || p.count < 1) return hipSuccess; \
        const int vec = p.bf16 ? 8 : 4; \
        if (p.count % vec == 0) { \
            if (p.bf16) hipLaunchKernelGGL(vkern<__bf16>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p); \
            else hipLaunchKernelGGL(vkern<float>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p); \
        } else { \
            if (p.bf16) hipLaunchKernelGGL(kern<__bf16>, ew_grid(p.count, n_active), dim3(256), 0, s, p); \
            else hipLaunchKernelGGL(kern<float>, ew_grid(p.count, n_active), dim3(256), 0, s, p); \
        } \
        return hipGetLastError(); }
HADFL_EW_VEC_LAUNCH(launch_add_fwd, add_fwd_vec_kernel, add_fwd_kernel)
HADFL_EW_VEC_LAUNCH(launch_pass_grad, pass_grad_vec_kernel, pass_grad_kernel)
#undef HADFL_EW_VEC_LAUNCH

hipError_t launch_maxpool_fwd(const EwParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1 || p.count < 1) return hipSuccess;
    const int vec = p.bf16 ? 8 : 4;
    if (p.C % vec == 0) {
        if (p.bf16) hipLaunchKernelGGL(maxpool_fwd_vec_kernel<__bf16>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p);
        else hipLaunchKernelGGL(maxpool_fwd_vec_kernel<float>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p);
    } else {
        if (p.bf16) hipLaunchKernelGGL(maxpool_fwd_kernel<__bf16>, ew_grid(p.count, n_active), dim3(256), 0, s, p);
        else hipLaunchKernelGGL(maxpool_fwd_kernel<float>, ew_grid(p.count, n_active), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_maxpool_bwd(const EwParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1 || p.count < 1) return hipSuccess;
    const int vec = p.bf16 ? 8 : 4;
    if (p.C % vec == 0) {
        if (p.bf16) hipLaunchKernelGGL(maxpool_bwd_vec_kernel<__bf16>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p);
        else hipLaunchKernelGGL(maxpool_bwd_vec_kernel<float>, ew_grid(p.count / vec, n_active), dim3(256), 0, s, p);
    } else {
        if (p.bf16) hipLaunchKernelGGL(maxpool_bwd_kernel<__bf16>, ew_grid(p.count, n_active), dim3(256), 0, s, p);
        else hipLaunchKernelGGL(maxpool_bwd_kernel<float>, ew_grid(p.count, n_active), dim3(256), 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_dense_small_fwd(const DenseSmallParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1 || p.rows < 1) return hipSuccess;
    if (p.bf16) hipLaunchKernelGGL((dense_small_fwd_kernel<16, __bf16>), dim3((unsigned)p.rows, (unsigned)n_active), dim3(256), 0, s, p);
    else hipLaunchKernelGGL((dense_small_fwd_kernel<16, float>), dim3((unsigned)p.rows, (unsigned)n_active), dim3(256), 0, s, p);
    return hipGetLastError();
}

namespace {
// channel vectors per workgroup: the largest power of two that is at most min(C / vec, 32)
int bn_cvb(int C, int vec) { int cv = C / vec, b = 1; while (b * 2 <= cv && b * 2 <= 32) b *= 2; return b; }
}  // namespace

hipError_t launch_bn_fwd(const BnParams& p0, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    BnParams p = p0;
    const int vec = p.bf16 ? 8 : 4;
    const dim3 block(256);
    if (p.C % vec == 0) {
        p.cvb = bn_cvb(p.C, vec);
        const int cgroups = (p.C / vec + p.cvb - 1) / p.cvb;
        const dim3 grid((unsigned)(p.chunks * cgroups), (unsigned)n_active), fgrid((unsigned)((p.C + 31) / 32), (unsigned)n_active);
        if (p.pool && (p.H % 2 != 0 || p.W % 2 != 0 || p.rows % 4 != 0 || !p.pool_out)) return hipErrorInvalidValue;
        if (p.bf16) {
            if (!p.stats_done) hipLaunchKernelGGL((bn_sums_vec_kernel<0, __bf16>), grid, block, 0, s, p);
            hipLaunchKernelGGL((bn_finalize_kernel<0, __bf16>), fgrid, block, 0, s, p);
            if (p.pool) hipLaunchKernelGGL(bn_apply_fwd_pool_vec_kernel<__bf16>, grid, block, 0, s, p);
            else hipLaunchKernelGGL(bn_apply_fwd_vec_kernel<__bf16>, grid, block, 0, s, p);
        } else {
            if (!p.stats_done) hipLaunchKernelGGL((bn_sums_vec_kernel<0, float>), grid, block, 0, s, p);
            hipLaunchKernelGGL((bn_finalize_kernel<0, float>), fgrid, block, 0, s, p);
            if (p.pool) hipLaunchKernelGGL(bn_apply_fwd_pool_vec_kernel<float>, grid, block, 0, s, p);
            else hipLaunchKernelGGL(bn_apply_fwd_vec_kernel<float>, grid, block, 0, s, p);
        }
        return hipGetLastError();
    }
    if (p.pool || p.stats_done) return hipErrorInvalidValue;  // the caller asks for these only where the vector kernels apply
    const dim3 grid((unsigned)(p.chunks * ((p.C + 63) / 64)), (unsigned)n_active);
    if (p.bf16) {
        hipLaunchKernelGGL((bn_reduce_kernel<0, __bf16>), grid, block, 0, s, p);
        hipLaunchKernelGGL((bn_reduce_kernel<1, __bf16>), grid, block, 0, s, p);
        hipLaunchKernelGGL(bn_apply_fwd_kernel<__bf16>, grid, block, 0, s, p);
    } else {
        hipLaunchKernelGGL((bn_reduce_kernel<0, float>), grid, block, 0, s, p);
        hipLaunchKernelGGL((bn_reduce_kernel<1, float>), grid, block, 0, s, p);
        hipLaunchKernelGGL(bn_apply_fwd_kernel<float>, grid, block, 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_bn_bwd(const BnParams& p0, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    BnParams p = p0;
    const int vec = p.bf16 ? 8 : 4;
    const dim3 block(256);
    if (p.C % vec == 0) {
        p.cvb = bn_cvb(p.C, vec);
        const int cgroups = (p.C / vec + p.cvb - 1) / p.cvb;
        const dim3 grid((unsigned)(p.chunks * cgroups), (unsigned)n_active), fgrid((unsigned)((p.C + 31) / 32), (unsigned)n_active);
        if (p.pool && (p.H % 2 != 0 || p.W % 2 != 0 || p.rows % 4 != 0 || !p.pool_g)) return hipErrorInvalidValue;
        if (p.bf16) {
            if (p.bwd_stats_done) {}                                  // the data gradient above left the sums
            else if (p.pool) hipLaunchKernelGGL(bn_sums_pool_vec_kernel<__bf16>, grid, block, 0, s, p);
            else hipLaunchKernelGGL((bn_sums_vec_kernel<1, __bf16>), grid, block, 0, s, p);
            hipLaunchKernelGGL((bn_finalize_kernel<1, __bf16>), fgrid, block, 0, s, p);
            if (p.pool) hipLaunchKernelGGL(bn_apply_bwd_pool_vec_kernel<__bf16>, grid, block, 0, s, p);
            else hipLaunchKernelGGL(bn_apply_bwd_vec_kernel<__bf16>, grid, block, 0, s, p);
        } else {
            if (p.bwd_stats_done) return hipErrorInvalidValue;       // only the bf16 data-gradient kernels leave them
            if (p.pool) hipLaunchKernelGGL(bn_sums_pool_vec_kernel<float>, grid, block, 0, s, p);
            else hipLaunchKernelGGL((bn_sums_vec_kernel<1, float>), grid, block, 0, s, p);
            hipLaunchKernelGGL((bn_finalize_kernel<1, float>), fgrid, block, 0, s, p);
            if (p.pool) hipLaunchKernelGGL(bn_apply_bwd_pool_vec_kernel<float>, grid, block, 0, s, p);
            else hipLaunchKernelGGL(bn_apply_bwd_vec_kernel<float>, grid, block, 0, s, p);
        }
        return hipGetLastError();
    }
    if (p.pool || p.bwd_stats_done) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(p.chunks * ((p.C + 63) / 64)), (unsigned)n_active);
    if (p.bf16) {
        hipLaunchKernelGGL((bn_reduce_kernel<2, __bf16>), grid, block, 0, s, p);
        hipLaunchKernelGGL(bn_apply_bwd_kernel<__bf16>, grid, block, 0, s, p);
    } else {
        hipLaunchKernelGGL((bn_reduce_kernel<2, float>), grid, block, 0, s, p);
        hipLaunchKernelGGL(bn_apply_bwd_kernel<float>, grid, block, 0, s, p);
    }
    return hipGetLastError();
}

hipError_t launch_softmax_ce(const LossParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    int threads = 64;
    while (threads < p.batch) threads *= 2;      // power of two for the tree; batch <= 1024 is checked at init
    if (p.bf16) hipLaunchKernelGGL(softmax_ce_kernel<__bf16>, dim3((unsigned)n_active), dim3((unsigned)threads), 0, s, p);
    else hipLaunchKernelGGL(softmax_ce_kernel<float>, dim3((unsigned)n_active), dim3((unsigned)threads), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_sgd(const SgdParams& p, int n_active, hipStream_t s)
{
    if (n_active < 1) return hipSuccess;
    if (p.n_seg < 0 || p.n_seg > kMaxSgdSegments) return hipErrorInvalidValue;
    long long n4 = 0;
    for (int k = 0; k < p.n_seg; ++k) {
        if (p.count[k] % 4 != 0 || p.first[k] % 4 != 0 || p.count[k] < 0) return hipErrorInvalidValue;
        n4 += p.count[k] / 4;
    }
    hipLaunchKernelGGL(sgd_kernel, ew_grid(n4 > 0 ? n4 : 1, n_active), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace hadfl
