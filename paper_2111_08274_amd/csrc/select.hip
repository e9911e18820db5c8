// Probability-based replica selection (paper Sec. 3.3) as one wavefront on the device.
// Built with -ffp-contract=off: every fp64 operation below is rounded on its own, so the result is a
// function of the inputs alone and any IEEE-754 implementation of the same written steps gives the same bits.
#include <climits>
#include <mutex>
#include <type_traits>

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

// Lane L receives the value of lane L - 1 (a wavefront-wide shift by one lane, DPP control wave_shr:1); lane 0, which
// has no lane below it, receives +0.0.
__device__ __forceinline__ double from_lane_below(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), 0x138, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), 0x138, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Running sums of one chunk of 64 non-negative values, one per lane, added strictly one after another in ascending
// lane order starting from `carry`: lane L ends with ((carry + v_0) + v_1) + ... + v_L, every addition rounded on its
// own.  Each pass hands every lane its lower neighbour's sum and adds the lane's own value (lane 0 adds carry + v_0
// to the +0.0 it is handed, which is exact).  A lane's sum is final one pass after its lower neighbour's is, and
// recomputing a final sum gives the same value again, so the passes need no lane test, no cross-lane read into
// scalar registers and no LDS.  On entry lanes below `first` must already hold their final sums in r (what they held
// after an earlier call whose values differed only at lanes >= first); the other lanes' r is ignored.  64 - first
// passes finish the chunk; they run in blocks of eight, the surplus passes change nothing.
__device__ __forceinline__ double ascending_sums(double mine, double carry, double r, int first)
{
    const double add = __lane_id() == 0 ? carry + mine : mine;
    for (int blk = (64 - first + 7) >> 3; blk > 0; --blk) {
#pragma unroll
        for (int i = 0; i < 8; ++i) r = from_lane_below(r) + add;
    }
    return r;
}

// Sixteen fp64 registers that a wave-uniform index can address (the compiler turns an indexed write into one
// register-relative move)
typedef double F16 __attribute__((ext_vector_type(16)));

template <typename V> __device__ __forceinline__ const V* versions_of(const SelectArgs& a);
template <> __device__ __forceinline__ const int* versions_of<int>(const SelectArgs& a) { return a.versions; }
template <> __device__ __forceinline__ const double* versions_of<double>(const SelectArgs& a) { return a.versions_f64; }

// V = int: versions are step counters; V = double: forecast (real-valued) versions (Sec. 3.2 feeding Sec. 3.3)
//
// What is serial in the rule and what is not.  The draws are sequential (draw t renormalises over the replicas that
// remain), and within a draw the total S and the running sums add f in ascending replica index, one rounded fp64
// addition after another: a chain of N dependent additions per draw that no reordering may touch, because the result
// is compared bit for bit.  Everything else is taken off that chain: the uniforms of all draws are computed up
// front (one Philox block per lane), f is computed once, and a step of the chain is a single v_add_f64 from
// registers when N <= 64 (a one-lane shift of the running sums and a v_add_f64 per step above that, ascending_sums).
// One wavefront on its own issues a dependent instruction only every 5 to 8 clocks, so what counts is the number of
// instructions on the path, and straight-line code that runs once is paid for in instruction fetches: the loops
// below are kept short rather than unrolled over all 64 lanes.
template <typename V>
__global__ __launch_bounds__(64) void select_kernel(SelectArgs a)
{
    constexpr bool kIntVersions = std::is_same<V, int>::value;
    __shared__ double s_sorted[kMaxReplicas];
    __shared__ double s_f[kMaxReplicas];
    __shared__ double s_u[kMaxReplicas];
    __shared__ unsigned char s_flag[kMaxReplicas];
    __shared__ V s_v[kMaxReplicas];
    __shared__ unsigned char s_av[kMaxReplicas];
    __shared__ long long s_key[kIntVersions ? kMaxReplicas : 1];
    const int lane = threadIdx.x, N = a.n;

    // versions and availability into LDS (one parallel load), then a rank-counting sort of the available versions:
    // rank(i) = #{available j : v_j < v_i or (v_j == v_i and j < i)}.
    const int chunks = (N + 63) / 64;
    for (int i = lane; i < chunks * 64; i += 64) {
        const bool on = i < N && (!a.avail || a.avail[i]);
        if (i < N) {
            s_v[i] = versions_of<V>(a)[i];
            s_av[i] = on ? 1 : 0;
            s_flag[i] = 0;
        }
        // step counters: (version, index) pairs are ordered by one integer key, version * 1024 + index; a replica
        // that is not available, or beyond N, gets the largest key and is counted before nobody
        if constexpr (kIntVersions) s_key[i] = on ? (long long)versions_of<V>(a)[i] * kMaxReplicas + i : LLONG_MAX;
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
    if constexpr (kIntVersions) {
        // every lane compares its own key with all keys, read from LDS at a wave-uniform address (a broadcast)
        for (int q = 0; q < chunks; ++q) {
            const int i = q * 64 + lane;
            const long long mine = s_key[i];
            na += __popcll(__ballot(mine != LLONG_MAX));
            int rank = 0;
            for (int j = 0; j < chunks * 64; j += 16) {
#pragma unroll
                for (int u = 0; u < 16; ++u) rank += s_key[j + u] < mine ? 1 : 0;
            }
            if (mine != LLONG_MAX) s_sorted[rank] = (double)s_v[i];
        }
    } else {
        // real-valued versions: lanes own elements i = 64q + lane and walk all j chunk by chunk with cross-lane reads
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
                    const int before = (int)(vj < vi) | ((int)(vj == vi) & (int)(j < i));
                    rank += before & (int)((mask >> k) & 1ull);
                }
            }
            if (i < N && s_av[i]) s_sorted[rank] = (double)vi;
        }
    }
    __syncthreads();
    // third quartile: linear interpolation at 0.75*(na-1)
    const double pos = 0.75 * (double)(na - 1);
    const int lo = (int)__builtin_floor(pos);
    const double frac = pos - (double)lo;
    double mu = s_sorted[lo];
    if (lo + 1 < na) mu = s_sorted[lo] + frac * (s_sorted[lo + 1] - s_sorted[lo]);
    __syncthreads();                                       // every lane has read the quartile before s_sorted is reused

    for (int i = lane; i < chunks * 64; i += 64) {         // f = +0.0 beyond N: the draws below need no bound test
        double f = 0.0;
        if (i < N && s_av[i]) {
            const double d = (double)s_v[i] - mu;
            double e = -(d * d) * 0.5;
            if (e < -690.0) e = -690.0;
            f = exp_neg(e);
        }
        s_f[i] = f;
        if (i < N) a.f[i] = f;
    }
    __syncthreads();

    // Sequential draws: draw t picks the first live replica whose running sum of f exceeds u_t * S, S the total over
    // the live replicas; dead replicas (picked, unavailable, or beyond N) add +0.0, which leaves a non-negative sum
    // unchanged.
    int n_picked = 0;
    if (chunks == 1) {
        // At most 64 replicas: the draws run from registers.  Lane L keeps g[j] = f_j for j <= L and +0.0 above, so
        // the plain chain ((0 + g[0]) + g[1]) + ... + g[63], the same instructions in every lane and no lane
        // waiting for another, leaves lane L with the running sum after replica L (the zeros above L change nothing)
        // and lane 63 with S.  A dependent v_add_f64 issues every 5 to 6 clocks, a quarter of what one step costs
        // when the running sum has to move to the next lane.  A picked replica is zeroed in every lane's g.
        F16 g0, g1, g2, g3, g4;
#pragma unroll
        for (int k = 0; k < 15; ++k) {
            g0[k] = k <= lane ? s_f[k] : 0.0;
            g1[k] = 15 + k <= lane ? s_f[15 + k] : 0.0;
            g2[k] = 30 + k <= lane ? s_f[30 + k] : 0.0;
            g3[k] = 45 + k <= lane ? s_f[45 + k] : 0.0;
            g4[k] = (k < 4 && 60 + k <= lane) ? s_f[60 + k] : 0.0;
        }
        g0[15] = 0.0; g1[15] = 0.0; g2[15] = 0.0; g3[15] = 0.0; g4[15] = 0.0;
        unsigned long long livemask = __ballot(s_f[lane] > 0.0);
        const unsigned long long could = livemask;
        const double my_u = lane < a.n_select ? s_u[lane] : 0.0;
        int my_pick = -1;
        for (int t = 0; t < a.n_select; ++t) {
            double q = 0.0;
#pragma unroll
            for (int k = 0; k < 15; ++k) q = q + g0[k];
#pragma unroll
            for (int k = 0; k < 15; ++k) q = q + g1[k];
#pragma unroll
            for (int k = 0; k < 15; ++k) q = q + g2[k];
#pragma unroll
            for (int k = 0; k < 15; ++k) q = q + g3[k];
#pragma unroll
            for (int k = 0; k < 4; ++k) q = q + g4[k];
            const double S = lane_value(q, 63);
            const double thr = lane_value(my_u, t) * S;
            const unsigned long long hit = __ballot(q > thr) & livemask;
            int pick = -1;
            if (hit) pick = __ffsll((long long)hit) - 1;
            else if (livemask) pick = 63 - __clzll(livemask);   // stays -1 only if no replica is left to draw from
            pick = __builtin_amdgcn_readfirstlane(pick);
            if (lane == t) my_pick = pick;
            // the picked replica leaves every lane's g: one register-indexed write per group, aimed at the spare
            // sixteenth element in the groups that do not hold it (and in all of them when nothing was picked)
            const int grp = pick >= 0 ? pick / 15 : 5, slot = pick - 15 * grp;
            g0[grp == 0 ? slot : 15] = 0.0;
            g1[grp == 1 ? slot : 15] = 0.0;
            g2[grp == 2 ? slot : 15] = 0.0;
            g3[grp == 3 ? slot : 15] = 0.0;
            g4[grp == 4 ? slot : 15] = 0.0;
            if (pick >= 0) {
                ++n_picked;
                livemask &= ~(1ull << pick);
            }
        }
        if (lane < a.n_select) a.selected[lane] = my_pick;
        if (lane < N) s_flag[lane] = (unsigned char)(((could & ~livemask) >> lane) & 1ull);
        __syncthreads();
    } else {
        // Sequential draws.  The wavefront walks the replicas in chunks of 64: every lane loads its own value once and
        // ends with the running sum after its element (ascending_sums), the last lane's carries into the next chunk.  The
        // total S is the last running sum; the pick is the first live element whose running sum exceeds u*S, found with one
        // compare and a ballot.  Dead elements (picked, unavailable, or beyond N) add +0.0, which leaves a non-negative sum
        // unchanged, so every chunk runs all 64 additions with no bound to test.
        //
        // Draw t + 1 differs from draw t in one element, the replica p picked last: the running sums below p are the same
        // additions of the same values and are kept (in LDS, s_sorted is free after the quartile), the chain restarts at p.
        int changed = 0;                                       // lowest replica whose running sum is not valid
        for (int t = 0; t < a.n_select; ++t) {
            const int c0 = changed >> 6;
            double run = c0 > 0 ? s_sorted[c0 * 64 - 1] : 0.0;
            for (int c = c0; c < chunks; ++c) {
                const int idx = c * 64 + lane;
                const bool live = idx < N && !s_flag[idx] && s_f[idx] > 0.0;
                const int first = c == c0 ? (changed & 63) : 0;
                const double prefix = ascending_sums(live ? s_f[idx] : 0.0, run, idx < N ? s_sorted[idx] : 0.0, first);
                if (idx < N) s_sorted[idx] = prefix;
                run = lane_value(prefix, 63);
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
            changed = pick >= 0 ? pick : N;                     // nothing left: later draws change nothing either
            __syncthreads();
        }
    }

    // aggregation weights a_k and the ascending list the aggregate kernel walks.  With unit terms the denominator is
    // the count itself (a sum of ones is exact); with f-weighted terms it adds the selected replicas' f in
    // ascending index, one after another, the same chain as above.
    double denom = (double)n_picked;
    if (a.weight_mode == 1) {
        denom = 0.0;
        for (int c = 0; c < chunks; ++c) {
            const int idx = c * 64 + lane;
            denom = lane_value(ascending_sums((idx < N && s_flag[idx]) ? s_f[idx] : 0.0, denom, 0.0, 0), 63);
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
