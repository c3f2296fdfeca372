// vt_layers.hip -- statistics that the element-wise fused layer + trainer-hook kernels read: per row
// for layer norm and softmax over rows too long or too short for the row-at-a-time kernels of
// vt_round_rowwise.hip (one wavefront per row, vt_rowstats.h), per column for batch norm.
#include "vt_device.h"
#include "vt_kernels.h"
#include "vt_rowstats.h"

#include <math.h>

namespace vt {

namespace {

__global__ __launch_bounds__(256) void layernorm_stats_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                              double eps, int variant, double *__restrict__ stat)
{
    const uint32_t lane = threadIdx.x & 63u, r = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (r >= rows) return;
    const stat_d2 st = norm_row_stats(x + (uint64_t)r * cols, cols, eps, variant, lane);
    if (lane == 0) *(stat_d2 *)(stat + 2 * (uint64_t)r) = st;
}

__global__ __launch_bounds__(256) void softmax_stats_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                            double scale, uint32_t period, int variant,
                                                            double *__restrict__ stat)
{
    const uint32_t lane = threadIdx.x & 63u, r = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (r >= rows) return;
    const stat_d2 st = softmax_row_stats(x + (uint64_t)r * cols, softmax_seen(r, cols, period), scale, variant, lane);
    if (lane == 0) *(stat_d2 *)(stat + 2 * (uint64_t)r) = st;
}

// ---- batch norm: statistics per column (channel) over all rows --------------------------------
// One read of the input.  The rows are cut into at most kSlabs slabs.  A workgroup owns one slab and
// up to 256 columns: its 256 threads are cpb columns x 256 / cpb row groups; row group g owns rows g,
// g + groups, ... of the slab for its column and takes them sixteen at a time (all sixteen loads in
// flight): count, mean and centred sum of squares of the sixteen from registers (two sweeps, as the
// definition has them), then merged into the thread's running triple by the pairwise update
//   n = na + nb,  d = mb - ma,  mean = ma + d nb / n,  M2 = M2a + M2b + d^2 na nb / n,
// which is exact in exact arithmetic and loses nothing to cancellation in floating point.  The row
// groups' triples are merged in a fixed order, and a second kernel merges the slabs' triples: one
// wavefront per column, every lane a run of consecutive slabs in order, then a fixed butterfly.
// Variant 0 walks rows, groups and slabs upwards, variant 1 downwards.
constexpr uint32_t kSlabs = 1024, kMomentRows = 16;

struct Moments { double n, mean, m2; };

__device__ __forceinline__ Moments merge(const Moments &a, const Moments &b)
{
    if (!(b.n > 0.0)) return a;
    if (!(a.n > 0.0)) return b;
    const double n = a.n + b.n;
    const double d = b.mean - a.mean, w = b.n / n;
    Moments r;
    r.n = n;
    r.mean = a.mean + d * w;
    r.m2 = (a.m2 + b.m2) + (d * d) * (a.n * w);
    return r;
}

// partial: [slab][3][cols] = (count, mean, M2) of the slab's rows per column
__global__ __launch_bounds__(256) void column_moments_kernel(const double *__restrict__ x, uint32_t rows, uint32_t cols,
                                                             uint32_t rows_per_slab, uint32_t cpb, int variant,
                                                             double *__restrict__ partial)
{
    __shared__ double part[3][256];
    const uint32_t t = threadIdx.x, cl = t % cpb, grp = t / cpb, groups = 256u / cpb;
    const uint32_t c = blockIdx.y * cpb + cl;
    const uint32_t r0 = blockIdx.x * rows_per_slab;
    const uint32_t r1 = r0 + rows_per_slab < rows ? r0 + rows_per_slab : rows;
    Moments run = {0.0, 0.0, 0.0};
    if (c < cols && r0 < rows) {
        const uint32_t mine = r1 - r0 > grp ? (r1 - r0 - grp + groups - 1) / groups : 0u;   // rows of this group
        for (uint32_t j0 = 0; j0 < mine; j0 += kMomentRows) {
            const uint32_t cnt = mine - j0 < kMomentRows ? mine - j0 : kMomentRows;
            double v[kMomentRows];
#pragma unroll
            for (uint32_t u = 0; u < kMomentRows; ++u) {
                const uint32_t j = j0 + (u < cnt ? u : 0u);
                const uint32_t r = r0 + grp + groups * (variant ? mine - 1 - j : j);
                v[u] = x[(uint64_t)r * cols + c];
            }
            double s = 0.0;
#pragma unroll
            for (uint32_t u = 0; u < kMomentRows; ++u)
                if (u < cnt) s = s + v[u];
            Moments blk;
            blk.n = (double)cnt;
            blk.mean = s / blk.n;
            double q = 0.0;
#pragma unroll
            for (uint32_t u = 0; u < kMomentRows; ++u)
                if (u < cnt) { const double d = v[u] - blk.mean; q = q + d * d; }
            blk.m2 = q;
            run = merge(run, blk);
        }
    }
    part[0][t] = run.n;
    part[1][t] = run.mean;
    part[2][t] = run.m2;
    __syncthreads();
    if (grp == 0 && c < cols) {
        Moments m = {0.0, 0.0, 0.0};
        for (uint32_t q = 0; q < groups; ++q) {
            const uint32_t at = (variant ? groups - 1 - q : q) * cpb + cl;
            m = merge(m, Moments{part[0][at], part[1][at], part[2][at]});
        }
        double *p = partial + (uint64_t)blockIdx.x * 3u * cols + c;
        p[0] = m.n;
        p[cols] = m.mean;
        p[2 * (uint64_t)cols] = m.m2;
    }
}

// stat[2c] = mean, stat[2c + 1] = 1 / sqrt(M2 / rows + eps); one wavefront per column
__global__ __launch_bounds__(256) void column_finish_kernel(const double *__restrict__ partial, uint32_t rows, uint32_t cols,
                                                            uint32_t slabs, double eps, int variant,
                                                            double *__restrict__ stat)
{
    const uint32_t lane = threadIdx.x & 63u, c = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (c >= cols) return;
    const uint32_t per = (slabs + 63u) / 64u;
    const uint32_t owner = variant ? 63u - lane : lane;              // variant 1: lane 0 holds the last run of slabs
    Moments m = {0.0, 0.0, 0.0};
    for (uint32_t i = 0; i < per; ++i) {
        const uint32_t q = owner * per + (variant ? per - 1 - i : i);
        if (q < slabs) {
            const double *p = partial + (uint64_t)q * 3u * cols + c;
            m = merge(m, Moments{p[0], p[cols], p[2 * (uint64_t)cols]});
        }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {                               // lane l absorbs lane l + o: runs stay in order
        Moments other;
        other.n = __shfl_down(m.n, o, 64);
        other.mean = __shfl_down(m.mean, o, 64);
        other.m2 = __shfl_down(m.m2, o, 64);
        if ((lane & (2u * o - 1u)) == 0) m = merge(m, other);
    }
    if (lane == 0) {
        stat[2 * (uint64_t)c] = m.mean;
        stat[2 * (uint64_t)c + 1] = 1.0 / sqrt(m.m2 / (double)rows + eps);
    }
}

}  // namespace

// per-row statistics, or per-column statistics followed by the slabs' partial sums
size_t layer_stat_bytes(uint64_t rows, uint64_t cols)
{
    const uint64_t row_wise = (rows * 16 + 255) / 256 * 256;
    const uint64_t col_wise = (cols * 16 + 255) / 256 * 256 + ((uint64_t)kSlabs * cols * 24 + 255) / 256 * 256;
    return (size_t)(row_wise > col_wise ? row_wise : col_wise);
}

hipError_t launch_layer_stats(const LayerArgs &g, uint64_t rows, hipStream_t s)
{
    if (rows == 0 || g.cols == 0) return hipSuccess;
    const double eps = g.eps;
    const int variant = g.variant;
    if (g.op == kLayerBatchNorm || g.op == kLayerBatchNormRelu) {
        double *stat = (double *)g.stat;
        double *partial = (double *)((char *)stat + ((uint64_t)g.cols * 16 + 255) / 256 * 256);
        const uint32_t cpb = g.cols <= 64 ? 64u : g.cols <= 128 ? 128u : 256u;
        const uint32_t per = (uint32_t)((rows + kSlabs - 1) / kSlabs);
        const uint32_t slabs = (uint32_t)((rows + per - 1) / per);
        const dim3 grid(slabs, (g.cols + cpb - 1) / cpb), block(256), fgrid((g.cols + 3) / 4);
        column_moments_kernel<<<grid, block, 0, s>>>(g.a, (uint32_t)rows, g.cols, per, cpb, variant, partial);
        column_finish_kernel<<<fgrid, block, 0, s>>>(partial, (uint32_t)rows, g.cols, slabs, eps, variant, stat);
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
