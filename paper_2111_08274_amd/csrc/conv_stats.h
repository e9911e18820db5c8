// Forward statistics of a batch norm from the epilogue of the convolution in front of it (shared by the bf16 and the fp32
// lean convolution kernels).
#pragma once
#include <hip/hip_runtime.h>

namespace hadfl {
namespace conv_stats {

typedef float f4 __attribute__((ext_vector_type(4)));

// Per-channel totals over a workgroup's output tile, for the forward statistics of a batch norm that follows the
// convolution.  ss[j][4g + e] / qq[..] are the lane's own sums (values, squares) over its rows for channel
// j*32 + 8g + 4*(lane >> 5) + e of the wave's column range.  Per wave the 32 row lanes of each half are added through a
// wave-private LDS area of 64 rows x kStatPitch(TN) floats: 16-byte writes, then lane (c4 = lane & 7, rg = lane >> 3) adds
// rows 8 rg .. 8 rg + 7 of four columns and two xor-shuffles join the four row groups of a half.  The WGM wave rows of
// the tile are then added in wave order through a second small area, and the waves of row 0 store the tile's entry:
// stat_slot[entry * 2 * N + n] = sum, [.. + N + n] = sum of squares.  Every order is fixed: the result is deterministic.
template <int TN> constexpr int kStatPitch = 16 * TN + 4;     // floats; 16 TN + 4 = 4 mod 32: conflict-free 16-byte accesses
template <int TN, int WGM, int WGN>
__device__ __forceinline__ void store_column_stats(const float (&ss)[TN][16], const float (&qq)[TN][16], float* smem_f, int wave, int lane,
                                                   float* stat_slot, int entry, int n_base, int N)
{
    constexpr int P = kStatPitch<TN>, NW = WGM * WGN;
    const int wm = wave / WGN;
    float* const area = smem_f + wave * (64 * P);
    float* const cross = smem_f + NW * (64 * P);              // [NW][2][16 TN][2 halves]
    float tot[2][4];
#pragma unroll
    for (int which = 0; which < 2; ++which) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const float (&v)[TN][16] = which ? qq : ss;
                *reinterpret_cast<f4*>(area + lane * P + j * 16 + 4 * g) = f4{v[j][4 * g], v[j][4 * g + 1], v[j][4 * g + 2], v[j][4 * g + 3]};
            }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        // TN = 2: 8 column quads x 8 row groups; TN = 1: 4 column quads, lanes with (lane & 7) >= 4 idle
        const int c4 = lane & 7, rg = lane >> 3;
        f4 t = {0.f, 0.f, 0.f, 0.f};
        if (c4 < 4 * TN) {
#pragma unroll
            for (int r = 0; r < 8; ++r) t += *reinterpret_cast<const f4*>(area + (rg * 8 + r) * P + c4 * 4);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = t[e];
            x += __shfl_xor(x, 8);                            // row groups rg ^ 1
            x += __shfl_xor(x, 16);                           // row groups rg ^ 2: lanes of one half now agree
            tot[which][e] = x;
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    // lanes with (rg & 3) == 0 hold the wave's totals of column quad c4 for half h = rg >> 2
    const int c4 = lane & 7, rg = lane >> 3, h = rg >> 2;
    const bool owner = (rg & 3) == 0 && c4 < 4 * TN;
    if (owner) {
#pragma unroll
        for (int which = 0; which < 2; ++which)
            *reinterpret_cast<f4*>(cross + ((wave * 2 + which) * (4 * TN) + c4) * 8 + h * 4) = f4{tot[which][0], tot[which][1], tot[which][2], tot[which][3]};
    }
    __syncthreads();
    if (owner && wm == 0) {
        const int wn = wave % WGN;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            f4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < WGM; ++r)
                a += *reinterpret_cast<const f4*>(cross + (((r * WGN + wn) * 2 + which) * (4 * TN) + c4) * 8 + h * 4);
            // column quad c4 of the area = (j, g) = (c4 / 4, c4 % 4): channels j*32 + 8g + 4h + {0..3}
            const int n = n_base + (c4 / 4) * 32 + 8 * (c4 % 4) + 4 * h;
            *reinterpret_cast<f4*>(stat_slot + (long long)entry * 2 * N + which * N + n) = a;
        }
    }
}
template <int TN, int WGM, int WGN> constexpr size_t kStatLdsBytes = ((size_t)WGM * WGN * 64 * kStatPitch<TN> + (size_t)WGM * WGN * 2 * 4 * TN * 8) * 4;

}  // namespace conv_stats
}  // namespace hadfl
