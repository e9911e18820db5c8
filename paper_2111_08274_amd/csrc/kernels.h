// Launch wrappers of the HIP kernels (host-callable), one per step of the cycle.
#pragma once
#include "hadfl_internal.h"

namespace hadfl {

// ---- selection (Sec. 3.3) -------------------------------------------------
struct SelectArgs {
    const int32_t* versions;       // [n] step counters, used when versions_f64 is null
    const double* versions_f64;    // [n] real-valued (forecast) versions, or null
    const uint8_t* avail;          // [n] or null
    int n, n_select, weight_mode;
    uint64_t seed, cycle;
    int32_t* selected;             // [n_select] draw order
    int32_t* sel_sorted;           // [n_select] ascending
    float* sel_weight;             // [n_select] weight of sel_sorted[i]
    uint8_t* flag;                 // [n]
    float* weights;                // [n]
    double* f;                     // [n]
};
hipError_t launch_select(const SelectArgs& a, hipStream_t s);
// The same kernel with f, sel_sorted and sel_weight taken from a static device array (at most kMaxReplicas replicas);
// allocates nothing.  a.f / a.sel_sorted / a.sel_weight are ignored.
hipError_t launch_select_static(SelectArgs a, hipStream_t s);
// Sec. 3.2: feed versions[n] into the smoothing states s1[n], s2[n] and write the forecast m cycles ahead to out[n]
hipError_t launch_predict(const int32_t* versions, double* s1, double* s2, double* out, int n, double alpha, int m,
                          int first, hipStream_t s);

// ---- aggregation + global synchronisation (Sec. 2.3, Algorithm 1) ----------
// agg[j] = sum_i sel_weight[i] * rows[sel_sorted[i]][j], i ascending; if n_bcast > 0 the result is also written
// to rows 0..n_bcast-1, or to rows bcast_list[0..n_bcast-1] when a list is given.  len is a multiple of 4 floats, all
// pointers 16-byte aligned.
hipError_t launch_aggregate(const float* rows, int64_t row_stride, int64_t len, const int32_t* sel_sorted,
                            const float* sel_weight, int n_select, float* agg, int n_bcast, float* rows_out,
                            const int32_t* bcast_list, hipStream_t s);

// ---- small utilities --------------------------------------------------------
hipError_t launch_copy_f32(const float* src, float* dst, int64_t count, hipStream_t s);
// dst[r*dst_stride + j] = src[j] for r < rows, j < count
hipError_t launch_bcast_rows(const float* src, float* dst, int64_t dst_stride, int64_t count, int rows, hipStream_t s);
hipError_t launch_fill_u32(uint32_t* dst, uint32_t v, int64_t count, hipStream_t s);

}  // namespace hadfl
