// Probability-based replica selection (paper Sec. 3.3) as one wavefront on the device.
// Built with -ffp-contract=off: every fp64 operation below is rounded on its own, so the result is a
// function of the inputs alone and any IEEE-754 implementation of the same written steps gives the same bits.
#include "kernels.h"

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

__global__ __launch_bounds__(64) void select_kernel(SelectArgs a)
{
    __shared__ double s_sorted[kMaxReplicas];
    __shared__ double s_f[kMaxReplicas];
    __shared__ unsigned char s_flag[kMaxReplicas];
    __shared__ int s_navail;
    const int lane = threadIdx.x, N = a.n;

    // versions of the available replicas, sorted ascending by rank counting
    if (lane == 0) {
        int c = 0;
        for (int k = 0; k < N; ++k) c += (!a.avail || a.avail[k]) ? 1 : 0;
        s_navail = c;
    }
    __syncthreads();
    const int na = s_navail;
    for (int i = lane; i < N; i += 64) {
        s_flag[i] = 0;
        if (a.avail && !a.avail[i]) continue;
        const int vi = a.versions[i];
        int rank = 0;
        for (int j = 0; j < N; ++j) {
            if (a.avail && !a.avail[j]) continue;
            const int vj = a.versions[j];
            rank += (vj < vi || (vj == vi && j < i)) ? 1 : 0;
        }
        s_sorted[rank] = (double)vi;
    }
    __syncthreads();
    // third quartile: linear interpolation at 0.75*(na-1)
    const double pos = 0.75 * (double)(na - 1);
    const int lo = (int)__builtin_floor(pos);
    const double frac = pos - (double)lo;
    double mu = s_sorted[lo];
    if (lo + 1 < na) mu = s_sorted[lo] + frac * (s_sorted[lo + 1] - s_sorted[lo]);

    for (int i = lane; i < N; i += 64) {
        double f = 0.0;
        if (!a.avail || a.avail[i]) {
            const double d = (double)a.versions[i] - mu;
            double e = -(d * d) * 0.5;
            if (e < -690.0) e = -690.0;
            f = exp_neg(e);
        }
        s_f[i] = f;
        a.f[i] = f;
    }
    __syncthreads();

    if (lane == 0) {
        for (int t = 0; t < a.n_select; ++t) {
            double S = 0.0;
            int last = -1;
            for (int k = 0; k < N; ++k)
                if (!s_flag[k] && s_f[k] > 0.0) { S += s_f[k]; last = k; }
            const U4 o = philox4x32_10(U4{(uint32_t)a.cycle, (uint32_t)(a.cycle >> 32), (uint32_t)t, 0u},
                                       (uint32_t)a.seed, (uint32_t)(a.seed >> 32));
            const unsigned long long bits = ((unsigned long long)o.y << 32) | o.x;
            const double u = (double)(bits >> 11) * 0x1.0p-53;
            const double thr = u * S;
            double run = 0.0;
            int pick = last;
            for (int k = 0; k < N; ++k) {
                if (s_flag[k] || !(s_f[k] > 0.0)) continue;
                run += s_f[k];
                if (run > thr) { pick = k; break; }
            }
            a.selected[t] = pick;
            s_flag[pick] = 1;
        }
        // aggregation weights a_k and the ascending list the aggregate kernel walks
        double denom = 0.0;
        for (int k = 0; k < N; ++k)
            if (s_flag[k]) denom += (a.weight_mode == 1) ? s_f[k] : 1.0;
        int c = 0;
        for (int k = 0; k < N; ++k) {
            float w = 0.f;
            if (s_flag[k]) {
                w = (float)(((a.weight_mode == 1) ? s_f[k] : 1.0) / denom);
                a.sel_sorted[c] = k;
                a.sel_weight[c] = w;
                ++c;
            }
            a.flag[k] = s_flag[k];
            a.weights[k] = w;
        }
    }
}

}  // namespace

hipError_t launch_select(const SelectArgs& a, hipStream_t s)
{
    hipLaunchKernelGGL(select_kernel, dim3(1), dim3(64), 0, s, a);
    return hipGetLastError();
}

}  // namespace hadfl
