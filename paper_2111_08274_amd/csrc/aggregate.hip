// Partial aggregation and global synchronisation (paper Sec. 2.3; Algorithm 1): a streaming weighted sum of the
// selected parameter rows.  HBM-bound: n_select rows are read once, the aggregate is written once, and in
// broadcast form every replica row is written once.  Unselected rows are never read.
#include "kernels.h"

namespace hadfl {
namespace {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr int kAggThreads = 256;
constexpr int kAggUnrollPlain = 2;  // float4 chunks per thread: 2*NP loads of 16 bytes in flight
constexpr int kAggUnrollBcast = 4;  // (the broadcast rows are written with plain stores: 4 % faster than non-temporal ones there)

// BCAST: the result is also written to n_bcast replica rows (a kernel name of its own in traces)
template <int NP, bool BCAST, int kAggUnroll = BCAST ? kAggUnrollBcast : kAggUnrollPlain>
__global__ __launch_bounds__(kAggThreads) void aggregate_kernel(
    const float* rows, int64_t row_stride, int64_t n4, const int32_t* __restrict__ sel,
    const float* __restrict__ wgt, int n_select, float* __restrict__ agg, int n_bcast, float* rows_out,
    const int32_t* __restrict__ bcast_list)
{
    const int np = NP > 0 ? NP : n_select;
    const int64_t base = ((int64_t)blockIdx.x * kAggUnroll) * kAggThreads + threadIdx.x;
    if (NP > 0) {
        const f4* src[NP > 0 ? NP : 1];
        float a[NP > 0 ? NP : 1];
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            src[i] = reinterpret_cast<const f4*>(rows + (int64_t)sel[i] * row_stride);
            a[i] = wgt[i];
        }
        f4 v[kAggUnroll][NP > 0 ? NP : 1];
#pragma unroll
        for (int u = 0; u < kAggUnroll; ++u) {
            const int64_t j = base + (int64_t)u * kAggThreads;
            if (j < n4) {
#pragma unroll
                for (int i = 0; i < NP; ++i) v[u][i] = __builtin_nontemporal_load(src[i] + j);
            }
        }
#pragma unroll
        for (int u = 0; u < kAggUnroll; ++u) {
            const int64_t j = base + (int64_t)u * kAggThreads;
            if (j < n4) {
                f4 acc = v[u][0] * a[0];
#pragma unroll
                for (int i = 1; i < NP; ++i) acc = acc + v[u][i] * a[i];
                __builtin_nontemporal_store(acc, reinterpret_cast<f4*>(agg) + j);
                if (BCAST)
                    for (int r = 0; r < n_bcast; ++r)
                        *(reinterpret_cast<f4*>(rows_out + (int64_t)(bcast_list ? bcast_list[r] : r) * row_stride) + j) = acc;
            }
        }
    } else {
        for (int u = 0; u < kAggUnroll; ++u) {
            const int64_t j = base + (int64_t)u * kAggThreads;
            if (j >= n4) continue;
            f4 acc = __builtin_nontemporal_load(reinterpret_cast<const f4*>(rows + (int64_t)sel[0] * row_stride) + j) * wgt[0];
            for (int i = 1; i < np; ++i)
                acc = acc + __builtin_nontemporal_load(reinterpret_cast<const f4*>(rows + (int64_t)sel[i] * row_stride) + j) * wgt[i];
            __builtin_nontemporal_store(acc, reinterpret_cast<f4*>(agg) + j);
            if (BCAST)
                for (int r = 0; r < n_bcast; ++r)
                    __builtin_nontemporal_store(acc, reinterpret_cast<f4*>(rows_out + (int64_t)(bcast_list ? bcast_list[r] : r) * row_stride) + j);
        }
    }
}

__global__ __launch_bounds__(256) void copy_kernel(const float* __restrict__ src, float* __restrict__ dst, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void bcast_rows_kernel(const float* __restrict__ src, float* __restrict__ dst,
                                                         int64_t dst_stride, int64_t count)
{
    float* d = dst + (int64_t)blockIdx.y * dst_stride;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) d[i] = src[i];
}

__global__ __launch_bounds__(256) void fill_kernel(uint32_t* dst, uint32_t v, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) dst[i] = v;
}

int grid_for(int64_t count, int per_block, int cap)
{
    int64_t b = (count + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > cap) b = cap;
    return (int)b;
}

}  // namespace

hipError_t launch_aggregate(const float* rows, int64_t row_stride, int64_t len, const int32_t* sel_sorted,
                            const float* sel_weight, int n_select, float* agg, int n_bcast, float* rows_out,
                            const int32_t* bcast_list, hipStream_t s)
{
    const int64_t n4 = len / 4;
    const int64_t per_block = (int64_t)kAggThreads * (n_bcast > 0 ? kAggUnrollBcast : kAggUnrollPlain);
    const dim3 grid((unsigned)((n4 + per_block - 1) / per_block)), block(kAggThreads);
#define HADFL_AGG(NP) do { \
        if (n_bcast > 0) hipLaunchKernelGGL((aggregate_kernel<NP, true>), grid, block, 0, s, rows, row_stride, n4, sel_sorted, \
                                            sel_weight, n_select, agg, n_bcast, rows_out, bcast_list); \
        else hipLaunchKernelGGL((aggregate_kernel<NP, false>), grid, block, 0, s, rows, row_stride, n4, sel_sorted, \
                                sel_weight, n_select, agg, n_bcast, rows_out, bcast_list); } while (0)
    switch (n_select) {
    case 1: HADFL_AGG(1); break;
    case 2: HADFL_AGG(2); break;
    case 3: HADFL_AGG(3); break;
    case 4: HADFL_AGG(4); break;
    case 5: HADFL_AGG(5); break;
    case 6: HADFL_AGG(6); break;
    case 7: HADFL_AGG(7); break;
    case 8: HADFL_AGG(8); break;
    default: HADFL_AGG(0); break;
    }
#undef HADFL_AGG
    return hipGetLastError();
}

hipError_t launch_copy_f32(const float* src, float* dst, int64_t count, hipStream_t s)
{
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for(count, 256, 4096)), dim3(256), 0, s, src, dst, count);
    return hipGetLastError();
}

hipError_t launch_bcast_rows(const float* src, float* dst, int64_t dst_stride, int64_t count, int rows, hipStream_t s)
{
    hipLaunchKernelGGL(bcast_rows_kernel, dim3(grid_for(count, 256, 2048), rows), dim3(256), 0, s, src, dst, dst_stride, count);
    return hipGetLastError();
}

hipError_t launch_fill_u32(uint32_t* dst, uint32_t v, int64_t count, hipStream_t s)
{
    hipLaunchKernelGGL(fill_kernel, dim3(grid_for(count, 256, 4096)), dim3(256), 0, s, dst, v, count);
    return hipGetLastError();
}

}  // namespace hadfl
