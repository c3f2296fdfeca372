// vt_layers.hip -- per-row statistics of the row-wise layers (layer norm, softmax) that the fused
// layer + trainer-hook kernels read: one wavefront per row, two sweeps over the row (the second
// one hits the cache), eight loads in flight per lane, FP64 throughout.
//
// Summation order: the row is cut into chunks of 512 columns; lane l owns columns l, l + 64, ...,
// l + 448 of each chunk and adds them to its partial sum chunk by chunk (variant 0: ascending
// columns, variant 1: descending), then the 64 partial sums are combined by a fixed butterfly
// (variant 0: strides 32, 16, ..., 1; variant 1: strides 1, 2, ..., 32).  Both orders are fixed, so
// a given variant always returns the same bits; the two variants differ in their low bits the
// way two GPU types do.
#include "vt_device.h"
#include "vt_kernels.h"

#include <math.h>

namespace vt {

namespace {

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

constexpr uint32_t kInFlight = 8, kChunkCols = 64 * kInFlight;

// Calls f(value) for every column c < lim of the row that belongs to this lane, in the variant's
// order; `load` maps a column to the value to accumulate.
template <class Load, class Fold>
__device__ __forceinline__ void sweep(uint32_t lim, uint32_t lane, int variant, Load load, Fold fold)
{
    const uint32_t chunks = (lim + kChunkCols - 1) / kChunkCols;
    for (uint32_t i = 0; i < chunks; ++i) {
        const uint32_t c0 = (variant ? chunks - 1 - i : i) * kChunkCols + lane;
        double v[kInFlight];
        bool in[kInFlight];
#pragma unroll
        for (uint32_t u = 0; u < kInFlight; ++u) {
            const uint32_t c = c0 + 64u * (variant ? kInFlight - 1 - u : u);
            in[u] = c < lim;
            v[u] = in[u] ? load(c) : 0.0;
        }
#pragma unroll
        for (uint32_t u = 0; u < kInFlight; ++u)
            if (in[u]) fold(v[u]);
    }
}

__global__ __launch_bounds__(256) void layernorm_stats_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                              double eps, int variant, double *__restrict__ stat)
{
    const uint32_t lane = threadIdx.x & 63u, r = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (r >= rows) return;
    const double *xr = x + (uint64_t)r * cols;
    double s = 0.0;
    sweep(cols, lane, variant, [&](uint32_t c) { return xr[c]; }, [&](double v) { s = s + v; });
    const double mean = wave_add(s, variant) / (double)cols;
    double q = 0.0;
    sweep(cols, lane, variant, [&](uint32_t c) { return xr[c]; }, [&](double v) { const double d = v - mean; q = q + d * d; });
    const double rstd = 1.0 / sqrt(wave_add(q, variant) / (double)cols + eps);
    if (lane == 0) {
        stat[2 * (uint64_t)r] = mean;
        stat[2 * (uint64_t)r + 1] = rstd;
    }
}

__global__ __launch_bounds__(256) void softmax_stats_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                            double scale, uint32_t period, int variant,
                                                            double *__restrict__ stat)
{
    const uint32_t lane = threadIdx.x & 63u, r = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (r >= rows) return;
    const double *xr = x + (uint64_t)r * cols;
    uint32_t seen = cols;                                           // columns 0 .. seen - 1 are visible
    if (period) seen = r % period + 1u < cols ? r % period + 1u : cols;
    double m = -INFINITY;
    sweep(seen, lane, 0, [&](uint32_t c) { return scale * xr[c]; }, [&](double z) { m = z > m ? z : m; });
    m = wave_max(m);
    double s = 0.0;
    sweep(seen, lane, variant, [&](uint32_t c) { return xr[c]; }, [&](double v) { s = s + exp(scale * v - m); });
    const double inv = 1.0 / wave_add(s, variant);
    if (lane == 0) {
        stat[2 * (uint64_t)r] = m;
        stat[2 * (uint64_t)r + 1] = inv;
    }
}

// ---- batch norm: statistics per column (channel) over all rows --------------------------------
// The rows are cut into kSlabs slabs.  A workgroup owns one slab and up to 256 columns: its 256
// threads are cpb columns x 256 / cpb row groups; row group g adds rows g, g + groups, ... of the slab
// for its column (variant 0: ascending, variant 1: descending), the groups are combined in a fixed
// order, and a second kernel adds the slabs' partial sums in a fixed order.  Two sweeps: the mean,
// then the centred squares.
constexpr uint32_t kSlabs = 1024;

template <bool CENTRED>
__global__ __launch_bounds__(256) void column_sums_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                          uint32_t rows_per_slab, uint32_t cpb,
                                                          const double *__restrict__ stat, int variant,
                                                          double *__restrict__ partial)
{
    __shared__ double part[256];
    const uint32_t t = threadIdx.x, cl = t % cpb, grp = t / cpb, groups = 256u / cpb;
    const uint32_t c = blockIdx.y * cpb + cl;
    const uint32_t r0 = blockIdx.x * rows_per_slab;
    const uint32_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    double acc = 0.0;
    if (c < cols && r0 < rows) {
        const double mean = CENTRED ? stat[2 * (uint64_t)c] : 0.0;
        const uint32_t mine = r1 - r0 > grp ? (r1 - r0 - grp + groups - 1) / groups : 0u;   // rows of this group
        for (uint32_t j0 = 0; j0 < mine; j0 += 4) {
            double v[4];
            bool in[4];
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u) {
                const uint32_t j = j0 + u;
                in[u] = j < mine;
                const uint32_t r = r0 + grp + groups * (variant ? mine - 1 - (in[u] ? j : 0) : (in[u] ? j : 0));
                v[u] = in[u] ? x[(uint64_t)r * cols + c] : 0.0;
            }
#pragma unroll
            for (uint32_t u = 0; u < 4; ++u)
                if (in[u]) {
                    if (CENTRED) { const double d = v[u] - mean; acc = acc + d * d; }
                    else acc = acc + v[u];
                }
        }
    }
    part[t] = acc;
    __syncthreads();
    if (grp == 0 && c < cols) {
        double s = 0.0;
        for (uint32_t q = 0; q < groups; ++q) s = s + part[(variant ? groups - 1 - q : q) * cpb + cl];
        partial[(uint64_t)blockIdx.x * cols + c] = s;
    }
}

// pass 0: stat[2c] = mean; pass 1: stat[2c + 1] = 1 / sqrt(var + eps)
__global__ __launch_bounds__(256) void column_finish_kernel(const double *__restrict__ partial, uint32_t rows, uint32_t cols,
                                                            uint32_t slabs, double eps, int pass, int variant,
                                                            double *__restrict__ stat)
{
    const uint32_t c = blockIdx.x * 256u + threadIdx.x;
    if (c >= cols) return;
    double s = 0.0;
    for (uint32_t q = 0; q < slabs; ++q) s = s + partial[(uint64_t)(variant ? slabs - 1 - q : q) * cols + c];
    if (pass == 0) stat[2 * (uint64_t)c] = s / (double)rows;
    else stat[2 * (uint64_t)c + 1] = 1.0 / sqrt(s / (double)rows + eps);
}

}  // namespace

// per-row statistics, or per-column statistics followed by the slabs' partial sums
size_t layer_stat_bytes(uint64_t rows, uint64_t cols)
{
    const uint64_t row_wise = (rows * 16 + 255) / 256 * 256;
    const uint64_t col_wise = (cols * 16 + 255) / 256 * 256 + ((uint64_t)kSlabs * cols * 8 + 255) / 256 * 256;
    return (size_t)(row_wise > col_wise ? row_wise : col_wise);
}

hipError_t launch_layer_stats(const LayerArgs &g, uint64_t rows, double eps, int variant, hipStream_t s)
{
    if (rows == 0 || g.cols == 0) return hipSuccess;
    if (g.op == kLayerBatchNorm || g.op == kLayerBatchNormRelu) {
        double *stat = (double *)g.stat;
        double *partial = (double *)((char *)stat + ((uint64_t)g.cols * 16 + 255) / 256 * 256);
        const uint32_t cpb = g.cols <= 64 ? 64u : g.cols <= 128 ? 128u : 256u;
        const uint32_t per = (uint32_t)((rows + kSlabs - 1) / kSlabs);
        const uint32_t slabs = (uint32_t)((rows + per - 1) / per);
        const dim3 grid(slabs, (g.cols + cpb - 1) / cpb), block(256), fgrid((g.cols + 255) / 256);
        column_sums_kernel<false><<<grid, block, 0, s>>>(g.a, (uint32_t)rows, g.cols, per, cpb, stat, variant, partial);
        column_finish_kernel<<<fgrid, block, 0, s>>>(partial, (uint32_t)rows, g.cols, slabs, eps, 0, variant, stat);
        column_sums_kernel<true><<<grid, block, 0, s>>>(g.a, (uint32_t)rows, g.cols, per, cpb, stat, variant, partial);
        column_finish_kernel<<<fgrid, block, 0, s>>>(partial, (uint32_t)rows, g.cols, slabs, eps, 1, variant, stat);
        return hipGetLastError();
    }
    if (g.op != kLayerNorm && g.op != kLayerSoftmax) return hipSuccess;
    const dim3 grid((uint32_t)((rows + 3) / 4)), block(256);
    if (g.op == kLayerNorm)
        layernorm_stats_kernel<<<grid, block, 0, s>>>(g.a, (uint32_t)rows, g.cols, eps, variant, (double *)g.stat);
    else
        softmax_stats_kernel<<<grid, block, 0, s>>>(g.a, (uint32_t)rows, g.cols, g.scale, g.period, variant,
                                                    (double *)g.stat);
    return hipGetLastError();
}

}  // namespace vt
