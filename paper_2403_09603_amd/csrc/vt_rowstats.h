// vt_rowstats.h -- statistics of one row of a row-wise layer (layer norm, softmax) by one wavefront:
// two sweeps over the row (the second one hits the cache), eight loads in flight per lane, FP64
// throughout.  The row-at-a-time kernels (vt_round_rowwise.hip) add up in the same order from
// registers, so a row's statistics have the same bits whichever kernel takes it.
//
// Summation order: lane l owns the column pairs (2l, 2l + 1), (128 + 2l, 128 + 2l + 1), ... of the
// row and adds them to its partial sum one after the other (variant 0: ascending columns, variant 1:
// descending), then the 64 partial sums are combined by a fixed butterfly (variant 0: strides 32,
// 16, ..., 1; variant 1: strides 1, 2, ..., 32).  Both orders are fixed, so
// a given variant always returns the same bits; the two variants differ in their low bits the
// way two GPU types do.
#pragma once
#include "vt_device.h"

#include <math.h>

namespace vt {

typedef double stat_d2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ double wave_add(double v, int variant)
{
    if (variant == 0) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v = v + __shfl_xor(v, o, 64);
    } else {
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) v = v + __shfl_xor(v, o, 64);
    }
    return v;
}

__device__ __forceinline__ double wave_max(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const double w = __shfl_xor(v, o, 64);
        v = w > v ? w : v;
    }
    return v;
}

constexpr uint32_t kRowInFlight = 8, kRowChunkCols = 128 * kRowInFlight;

// Calls fold(column, value) for every column c < lim of the row that belongs to this lane, in the
// variant's order.  Rows that start on a 16-byte boundary are read two values per load.
template <class Fold>
__device__ __forceinline__ void row_sweep(const double *__restrict__ xr, uint32_t lim, uint32_t lane, int variant, Fold fold)
{
    const bool aligned = ((uintptr_t)xr & 15u) == 0;                 // the same for the whole wave
    const uint32_t chunks = (lim + kRowChunkCols - 1) / kRowChunkCols;
    for (uint32_t i = 0; i < chunks; ++i) {
        const uint32_t c0 = (variant ? chunks - 1 - i : i) * kRowChunkCols + 2u * lane;
        stat_d2 v[kRowInFlight];
#pragma unroll
        for (uint32_t u = 0; u < kRowInFlight; ++u) {
            const uint32_t c = c0 + 128u * (variant ? kRowInFlight - 1 - u : u);
            if (aligned && c + 1 < lim) v[u] = *(const stat_d2 *)(xr + c);
            else {
                v[u].x = c < lim ? xr[c] : 0.0;
                v[u].y = c + 1 < lim ? xr[c + 1] : 0.0;
            }
        }
#pragma unroll
        for (uint32_t u = 0; u < kRowInFlight; ++u) {
            const uint32_t c = c0 + 128u * (variant ? kRowInFlight - 1 - u : u);
            if (variant == 0) {
                if (c < lim) fold(c, v[u].x);
                if (c + 1 < lim) fold(c + 1, v[u].y);
            } else {
                if (c + 1 < lim) fold(c + 1, v[u].y);
                if (c < lim) fold(c, v[u].x);
            }
        }
    }
}

// (mean, 1 / sqrt(variance + eps)) of xr[0 .. cols): the same pair in every lane
__device__ __forceinline__ stat_d2 norm_row_stats(const double *__restrict__ xr, uint32_t cols, double eps, int variant,
                                                  uint32_t lane)
{
    double s = 0.0;
    row_sweep(xr, cols, lane, variant, [&](uint32_t, double v) { s = s + v; });
    const double mean = wave_add(s, variant) / (double)cols;
    double q = 0.0;
    row_sweep(xr, cols, lane, variant, [&](uint32_t, double v) { const double d = v - mean; q = q + d * d; });
    stat_d2 st;
    st.x = mean;
    st.y = 1.0 / sqrt(wave_add(q, variant) / (double)cols + eps);
    return st;
}

// (max, 1 / sum of exp(scale x - max)) over the visible columns 0 .. seen - 1: the same pair in every lane
__device__ __forceinline__ stat_d2 softmax_row_stats(const double *__restrict__ xr, uint32_t seen, double scale, int variant,
                                                     uint32_t lane)
{
    double m = -INFINITY;
    row_sweep(xr, seen, lane, 0, [&](uint32_t, double v) { const double z = scale * v; m = z > m ? z : m; });
    m = wave_max(m);
    double s = 0.0;
    row_sweep(xr, seen, lane, variant, [&](uint32_t, double v) { s = s + exp(scale * v - m); });
    stat_d2 st;
    st.x = m;
    st.y = 1.0 / wave_add(s, variant);
    return st;
}

// columns of row r that a softmax with causal period `period` sees (0 = all)
__device__ __forceinline__ uint32_t softmax_seen(uint32_t r, uint32_t cols, uint32_t period)
{
    if (!period) return cols;
    const uint32_t rem = r % period;
    return rem + 1u < cols ? rem + 1u : cols;
}

}  // namespace vt
