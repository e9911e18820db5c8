// Probability-based replica selection (paper Sec. 3.3) as one wavefront on the device.
// Built with -ffp-contract=off: every fp64 operation below is rounded on its own, so the result is a
// function of the inputs alone and any IEEE-754 implementation of the same written steps gives the same bits.
#include <mutex>

#include "kernels.h"

// Working memory of hadfl_select_static, the selection for callers that cannot allocate device memory: the selection
// function's values f[kMaxReplicas] (fp64), then the ascending list of the selected replicas and their weights.
// Every GPU the library runs on holds its own copy until the process ends.  Host code never passes this name to a
// kernel: it is a host-side stand-in, the device address comes from hipGetSymbolAddress (static_scratch below).
constexpr size_t kStaticScratchBytes = hadfl::kMaxReplicas * (sizeof(double) + sizeof(int32_t) + sizeof(float));
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace hadfl {
namespace {

struct U4 { uint32_t x, y, z, w; };

// Philox4x32-10 (Salmon et al., SC'11).
__device__ U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t lo0 = 0xD2511F53u * c.x, hi0 = __umulhi(0xD2511F53u, c.x);
        const uint32_t lo1 = 0xCD9E8D57u * c.z, hi1 = __umulhi(0xCD9E8D57u, c.z);
        c = U4{hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0};
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c;
}

// exp(x), x in [-690, 0]: n = nearest integer to x*log2(e); r = (x - n*ln2_hi) - n*ln2_lo (two-constant
// reduction, n*ln2_hi exact); Taylor polynomial of degree 13 by Horner; multiply by 2^n built in the exponent field.
__device__ double exp_neg(double x)
{
    const double c[14] = {1.0, 1.0, 1.0 / 2.0, 1.0 / 6.0, 1.0 / 24.0, 1.0 / 120.0, 1.0 / 720.0, 1.0 / 5040.0,
                          1.0 / 40320.0, 1.0 / 362880.0, 1.0 / 3628800.0, 1.0 / 39916800.0,
                          1.0 / 479001600.0, 1.0 / 6227020800.0};
    const double n = __builtin_rint(x * 0x1.71547652b82fep+0);
    const double r = (x - n * 0x1.62e42feep-1) - n * 0x1.a39ef35793c76p-33;
    double p = c[13];
#pragma unroll
    for (int i = 12; i >= 0; --i) p = p * r + c[i];
    const long long e = (long long)n + 1023;
    if (e < 1) return 0.0;
    return p * __longlong_as_double(e << 52);
}

// value held by lane k of the wavefront (k is wave-uniform at every call site)
__device__ __forceinline__ double lane_value(double v, int k)
{
    const int lo = __builtin_amdgcn_readlane(__double2loint(v), k);
    const int hi = __builtin_amdgcn_readlane(__double2hiint(v), k);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ int lane_value(int v, int k) { return __builtin_amdgcn_readlane(v, k); }

template <typename V> __device__ __forceinline__ const V* versions_of(const SelectArgs& a);
template <> __device__ __forceinline__ const int* versions_of<int>(const SelectArgs& a) { return a.versions; }
template <> __device__ __forceinline__ const double* versions_of<double>(const SelectArgs& a) { return a.versions_f64; }

// V = int: versions are step counters; V = double: forecast (real-valued) versions (Sec. 3.2 feeding Sec. 3.3)
//
// What is serial in the rule and what is not.  The draws are sequential (draw t renormalises over the replicas that
// remain), and within a draw the total S and the running sums add f in ascending replica index, one rounded fp64
// addition after another: a chain of N dependent additions per draw that no reordering may touch, because the result
// is compared bit for bit.  Everything else is taken off that chain: the uniforms of all draws are computed up
// front (one Philox block per lane), f is computed once, and inside a chunk of 64 replicas the chain is a fully
// unrolled run of v_add_f64 whose operands (cross-lane reads of the lanes' own values) do not depend on the chain.
template <typename V>
__global__ __launch_bounds__(64) void select_kernel(SelectArgs a)
{
    __shared__ double s_sorted[kMaxReplicas];
    __shared__ double s_f[kMaxReplicas];
    __shared__ double s_u[kMaxReplicas];
    __shared__ unsigned char s_flag[kMaxReplicas];
    __shared__ V s_v[kMaxReplicas];
    __shared__ unsigned char s_av[kMaxReplicas];
    const int lane = threadIdx.x, N = a.n;

    // versions and availability into LDS (one parallel load), then a rank-counting sort of the available versions:
    // rank(i) = #{available j : v_j < v_i or (v_j == v_i and j < i)}.  Lanes own elements i = 64q + lane and walk all j
    // chunk by chunk with cross-lane reads, so no step waits on memory.
    const int chunks = (N + 63) / 64;
    for (int i = lane; i < N; i += 64) {
        s_v[i] = versions_of<V>(a)[i];
        s_av[i] = (!a.avail || a.avail[i]) ? 1 : 0;
        s_flag[i] = 0;
    }
    // the uniform of every draw: counter (cycle_lo, cycle_hi, draw, 0), key = seed, 53 bits of the first two words
    for (int t = lane; t < a.n_select; t += 64) {
        const U4 o = philox4x32_10(U4{(uint32_t)a.cycle, (uint32_t)(a.cycle >> 32), (uint32_t)t, 0u},
                                   (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
        const unsigned long long bits = ((unsigned long long)o.y << 32) | o.x;
        s_u[t] = (double)(bits >> 11) * 0x1.0p-53;
    }
    __syncthreads();
    int na = 0;
    for (int q = 0; q < chunks; ++q) {
        const int i = q * 64 + lane;
        const V vi = i < N ? s_v[i] : V(0);
        int rank = 0;
        na = 0;
        for (int c = 0; c < chunks; ++c) {
            const int idx = c * 64 + lane;
            const V vjm = idx < N ? s_v[idx] : V(0);
            const unsigned long long mask = __ballot(idx < N && s_av[idx]);
            na += __popcll(mask);
#pragma unroll
            for (int k = 0; k < 64; ++k) {
                const V vj = lane_value(vjm, k);
                const int j = c * 64 + k;
                const bool bj = (mask >> k) & 1ull;
                rank += (bj && (vj < vi || (vj == vi && j < i))) ? 1 : 0;
            }
        }
        if (i < N && s_av[i]) s_sorted[rank] = (double)vi;
    }
    __syncthreads();
    // third quartile: linear interpolation at 0.75*(na-1)
    const double pos = 0.75 * (double)(na - 1);
    const int lo = (int)__builtin_floor(pos);
    const double frac = pos - (double)lo;
    double mu = s_sorted[lo];
    if (lo + 1 < na) mu = s_sorted[lo] + frac * (s_sorted[lo + 1] - s_sorted[lo]);
    __syncthreads();                                       // every lane has read the quartile before s_sorted is reused

    for (int i = lane; i < N; i += 64) {
        double f = 0.0;
        if (s_av[i]) {
            const double d = (double)s_v[i] - mu;
            double e = -(d * d) * 0.5;
            if (e < -690.0) e = -690.0;
            f = exp_neg(e);
        }
        s_f[i] = f;
        a.f[i] = f;
    }
    __syncthreads();

    // Sequential draws.  The wavefront walks the replicas in chunks of 64: every lane loads its own value once, then
    // all lanes step through the chunk together, and lane k keeps the running sum after element k.  The total S is the
    // last running sum; the pick is the first live element whose running sum exceeds u*S, found with one compare and a
    // ballot.  Dead elements (picked, unavailable, or beyond N) add +0.0, which leaves a non-negative sum unchanged, so
    // every chunk runs all 64 additions with no bound to test.
    int n_picked = 0;
    for (int t = 0; t < a.n_select; ++t) {
        double run = 0.0;
        for (int c = 0; c < chunks; ++c) {
            const int idx = c * 64 + lane;
            const bool live = idx < N && !s_flag[idx] && s_f[idx] > 0.0;
            const double mine = live ? s_f[idx] : 0.0;
            double prefix = 0.0;
#pragma unroll
            for (int k = 0; k < 64; ++k) {
                run = run + lane_value(mine, k);
                prefix = (lane == k) ? run : prefix;
            }
            if (idx < N) s_sorted[idx] = prefix;          // s_sorted is free after the quartile: reuse as prefix store
        }
        const double S = run;
        const double thr = s_u[t] * S;
        int pick = -1, last = -1;
        for (int c = 0; c < chunks; ++c) {
            const int idx = c * 64 + lane;
            const bool live = idx < N && !s_flag[idx] && s_f[idx] > 0.0;
            const unsigned long long lm = __ballot(live);
            const unsigned long long hit = __ballot(live && s_sorted[idx < N ? idx : 0] > thr);
            if (lm) last = c * 64 + 63 - __clzll(lm);
            if (pick < 0 && hit) pick = c * 64 + __ffsll((long long)hit) - 1;
        }
        if (pick < 0) pick = last;                         // stays -1 only if no replica is left to draw from
        n_picked += pick >= 0 ? 1 : 0;
        __syncthreads();
        if (lane == 0) { a.selected[t] = pick; if (pick >= 0) s_flag[pick] = 1; }
        __syncthreads();
    }

    // aggregation weights a_k and the ascending list the aggregate kernel walks.  With unit terms the denominator is
    // the count itself (a sum of ones is exact); with f-weighted terms it adds the selected replicas' f in
    // ascending index, one after another, the same chain as above.
    double denom = (double)n_picked;
    if (a.weight_mode == 1) {
        denom = 0.0;
        for (int c = 0; c < chunks; ++c) {
            const int idx = c * 64 + lane;
            const double mine = (idx < N && s_flag[idx]) ? s_f[idx] : 0.0;
#pragma unroll
            for (int k = 0; k < 64; ++k) denom = denom + lane_value(mine, k);
        }
    }
    int before = 0;                                        // selected replicas in earlier chunks
    for (int c = 0; c < chunks; ++c) {
        const int idx = c * 64 + lane;
        const bool on = idx < N && s_flag[idx];
        const unsigned long long m = __ballot(on);
        if (idx < N) {
            float w = 0.f;
            if (on) {
                w = (float)(((a.weight_mode == 1) ? s_f[idx] : 1.0) / denom);
                const int pos = before + __popcll(m & ((1ull << lane) - 1ull));
                a.sel_sorted[pos] = idx;
                a.sel_weight[pos] = w;
            }
            a.flag[idx] = s_flag[idx];
            a.weights[idx] = w;
        }
        before += __popcll(m);
    }
}

// Version forecast (Sec. 3.2): double exponential smoothing of every replica's version series.
//   s1 <- alpha*v + (1-alpha)*s1;  s2 <- alpha*s1 + (1-alpha)*s2   (both start at the first observation)
//   forecast(m) = (2*s1 - s2) + alpha/(1-alpha)*(s1 - s2)*m
__global__ __launch_bounds__(64) void predict_kernel(const int32_t* versions, double* s1, double* s2, double* out, int n,
                                                     double alpha, int m, int first)
{
    for (int i = threadIdx.x; i < n; i += 64) {
        const double v = (double)versions[i];
        double a1, a2;
        if (first) { a1 = v; a2 = v; }
        else {
            a1 = alpha * v + (1.0 - alpha) * s1[i];
            a2 = alpha * a1 + (1.0 - alpha) * s2[i];
        }
        s1[i] = a1; s2[i] = a2;
        const double level = 2.0 * a1 - a2;
        const double trend = alpha / (1.0 - alpha) * (a1 - a2);
        out[i] = level + trend * (double)m;
    }
}

}  // namespace

hipError_t launch_predict(const int32_t* versions, double* s1, double* s2, double* out, int n, double alpha, int m,
                          int first, hipStream_t s)
{
    hipLaunchKernelGGL(predict_kernel, dim3(1), dim3(64), 0, s, versions, s1, s2, out, n, alpha, m, first);
    return hipGetLastError();
}

// Device address of this GPU's copy of `scratch`, looked up once per device with that device current.
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(unsigned char** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
    return hipSuccess;
}
}  // namespace

hipError_t launch_select_static(SelectArgs a, hipStream_t s)
{
    if (a.n < 1 || a.n > kMaxReplicas || a.n_select < 1 || a.n_select > a.n) return hipErrorInvalidValue;
    unsigned char* base = nullptr;
    const hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return e;
    // the kernel writes every entry of these three before it reads it, so nothing has to be cleared between calls
    a.f = reinterpret_cast<double*>(base);
    a.sel_sorted = reinterpret_cast<int32_t*>(base + kMaxReplicas * sizeof(double));
    a.sel_weight = reinterpret_cast<float*>(base + kMaxReplicas * (sizeof(double) + sizeof(int32_t)));
    return launch_select(a, s);
}

hipError_t launch_select(const SelectArgs& a, hipStream_t s)
{
    if (a.versions_f64) hipLaunchKernelGGL(select_kernel<double>, dim3(1), dim3(64), 0, s, a);
    else hipLaunchKernelGGL(select_kernel<int>, dim3(1), dim3(64), 0, s, a);
    return hipGetLastError();
}

}  // namespace hadfl
