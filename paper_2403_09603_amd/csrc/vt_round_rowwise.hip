// vt_round_rowwise.hip -- layer norm and softmax fused with the trainer hook, a row at a time in
// registers (gfx950, wave64): the input is read from memory once, the statistics of a row, its FP64
// outputs (softmax: one exponential per value, kept between the sum and the division), their
// rounding and their log decisions all come from the same registers, and nothing but the outputs is
// written.
//
// A wavefront owns five consecutive rows: five rows are a whole number of bytes of the packed
// ternary log (five outputs per byte) whatever the row length, so a wave's part of either log format
// is its own.  Lane l holds the column pairs (2 l, 2 l + 1), (128 + 2 l, ...), ... of the current row
// (up to 128 U columns, 16-byte loads and 8-byte stores; the next row is already on its way).  The sums run over a lane's columns upwards (variant 0) or downwards (variant 1) and
// across the lanes by the butterfly of vt_rowstats.h: the summation order, and with it every bit, is
// that of the stand-alone statistics kernel followed by the element-wise pass.  Packed log: codes go
// to LDS by output position and every lane packs four bytes (twenty outputs) at a time.  Index-list
// log: the entries are compacted per wave in LDS by ballots (lane by lane and pair by pair a group of
// 128 columns is in output order), and a workgroup of four waves is one tile of the scanner protocol
// (vt_scan.h).
#include "vt_device.h"
#include "vt_kernels.h"
#include "vt_rowstats.h"
#include "vt_scan.h"

#include <math.h>

namespace vt {

namespace {

constexpr int kRwWaves = 4;
constexpr uint32_t kRwRows = 5;               // rows per wave
constexpr uint32_t kRwSlots = 256, kRwSlotStride = 8;   // the packed-log kernels' spread counters (vt_round_dense.hip)

typedef double d2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

// lane l takes the column pairs (128 u + 2 l, 128 u + 2 l + 1); columns past the row read as 0
template <int U>
__device__ __forceinline__ void load_row(const double *__restrict__ xr, uint32_t cols, uint32_t lane, d2 (&v)[U])
{
    const bool aligned = ((uintptr_t)xr & 15u) == 0;        // the same for the whole wave
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t c = 128u * u + 2u * lane;
        if (aligned && c + 1 < cols) v[u] = __builtin_nontemporal_load((const d2 *)(xr + c));
        else {
            v[u].x = c < cols ? __builtin_nontemporal_load(xr + c) : 0.0;
            v[u].y = c + 1 < cols ? __builtin_nontemporal_load(xr + c + 1) : 0.0;
        }
    }
}

// sum of f(value) over this lane's columns below lim, in the variant's order (as row_sweep has it)
template <int U, class F>
__device__ __forceinline__ double lane_sum(const d2 (&v)[U], uint32_t lim, uint32_t lane, int variant, F f)
{
    double s = 0.0;
    if (variant == 0) {
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = 128u * u + 2u * lane;
            if (c < lim) s = s + f(v[u].x);
            if (c + 1 < lim) s = s + f(v[u].y);
        }
    } else {
#pragma unroll
        for (int u = U - 1; u >= 0; --u) {
            const uint32_t c = 128u * u + 2u * lane;
            if (c + 1 < lim) s = s + f(v[u].y);
            if (c < lim) s = s + f(v[u].x);
        }
    }
    return s;
}

// The layer's outputs of one row, in place: v[u] becomes the FP64 outputs of the lane's columns.
template <int OP, int U>
__device__ __forceinline__ void row_outputs(const LayerArgs &g, uint32_t r, uint32_t lane, d2 (&v)[U])
{
    const uint32_t cols = g.cols;
    if (OP == kLayerNorm) {
        const double mean = wave_add(lane_sum(v, cols, lane, g.variant, [](double x) { return x; }), g.variant) / (double)cols;
        const double q = lane_sum(v, cols, lane, g.variant, [&](double x) { const double d = x - mean; return d * d; });
        const double rstd = 1.0 / sqrt(wave_add(q, g.variant) / (double)cols + g.eps);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = 128u * u + 2u * lane;
            if (c < cols) {
                double o = (v[u].x - mean) * rstd;
                if (g.gamma) o = o * g.gamma[c];
                if (g.beta) o = o + g.beta[c];
                v[u].x = o;
            }
            if (c + 1 < cols) {
                double o = (v[u].y - mean) * rstd;
                if (g.gamma) o = o * g.gamma[c + 1];
                if (g.beta) o = o + g.beta[c + 1];
                v[u].y = o;
            }
        }
    } else {
        const uint32_t seen = softmax_seen(r, cols, g.period);
        double m = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = 128u * u + 2u * lane;
            if (c < seen) { const double z = g.scale * v[u].x; m = z > m ? z : m; }
            if (c + 1 < seen) { const double z = g.scale * v[u].y; m = z > m ? z : m; }
        }
        m = wave_max(m);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = 128u * u + 2u * lane;
            if (c < seen) v[u].x = exp(g.scale * v[u].x - m);
            if (c + 1 < seen) v[u].y = exp(g.scale * v[u].y - m);
        }
        const double inv = 1.0 / wave_add(lane_sum(v, seen, lane, g.variant, [](double p) { return p; }), g.variant);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint32_t c = 128u * u + 2u * lane;
            v[u].x = c < seen ? v[u].x * inv : 0.0;
            v[u].y = c + 1 < seen ? v[u].y * inv : 0.0;
        }
    }
}

// DENSE: tlog / slots are used; otherwise the scanner's arguments (workgroup 0 is the scanner).
template <int OP, int U, bool K0, bool DENSE>
__global__ __launch_bounds__(256) void rowwise_kernel(const LayerArgs g, uint32_t rows, uint32_t thr, uint32_t k,
                                                      float *__restrict__ y, uint8_t *__restrict__ tlog,
                                                      uint64_t *__restrict__ slots, uint64_t *__restrict__ st,
                                                      uint32_t tiles, uint32_t *__restrict__ err,
                                                      uint32_t *__restrict__ idx, uint32_t *__restrict__ dir, uint64_t cap,
                                                      uint64_t *__restrict__ count)
{
    constexpr uint32_t kWaveOut = kRwRows * 128u * U;       // most outputs of one wave
    constexpr bool PREFETCH = true;
    static_assert(kWaveOut <= 0x8000u, "an entry holds a 15-bit position");
    __shared__ __attribute__((aligned(16))) uint8_t smem[kRwWaves * kWaveOut * (DENSE ? 1 : 2)];
    __shared__ uint32_t s_wc[8];                            // entries per wave (scanner: its 8 words of scratch)
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
    uint32_t tile = blockIdx.x;
    if (!DENSE) {
        if (blockIdx.x == 0) {
            if (tid < (uint32_t)kScannerThreads) scanner(st, tiles, err, count, s_wc);
            return;
        }
        tile = blockIdx.x - 1;
    }
    const uint32_t cols = g.cols;
    const uint32_t group = tile * kRwWaves + wv;
    const uint32_t r0 = group * kRwRows;
    const uint32_t nrows = r0 < rows ? (rows - r0 < kRwRows ? rows - r0 : kRwRows) : 0u;
    uint8_t *codes = smem + wv * kWaveOut;
    uint16_t *ent = (uint16_t *)smem + wv * kWaveOut;
    uint32_t wcount = 0;                                    // logged outputs of this wave (sparse: entries written)

    d2 cur[U], nxt[PREFETCH ? U : 1];
    if (nrows) load_row<U>(g.a + (uint64_t)r0 * cols, cols, lane, cur);
    for (uint32_t j = 0; j < nrows; ++j) {
        const uint32_t r = r0 + j;
        if constexpr (PREFETCH) {
            if (j + 1 < nrows) load_row<U>(g.a + (uint64_t)(r + 1) * cols, cols, lane, nxt);
        }
        row_outputs<OP, U>(g, r, lane, cur);
        const uint64_t e_row = (uint64_t)r * cols;
        const bool y_pairs = (((uintptr_t)(y + e_row)) & 7u) == 0;            // uniform: 8-byte stores are aligned
        const bool y64_pairs = g.y64 && (((uintptr_t)g.y64 + 8u * e_row) & 15u) == 0;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (128u * u < cols) {                          // uniform: the row has columns in this group of 128
                const uint32_t c = 128u * u + 2u * lane;
                const bool va = c < cols, vb = c + 1 < cols;
                const double oa = va ? cur[u].x : 1.0, ob = vb ? cur[u].y : 1.0;      // 1.0 is never logged
                const Rounded ra = round_decide<K0>(oa, thr, k), rb = round_decide<K0>(ob, thr, k);
                if (vb && y_pairs) {
                    f2 o;
                    o.x = __uint_as_float(ra.ybits);
                    o.y = __uint_as_float(rb.ybits);
                    __builtin_nontemporal_store(o, (f2 *)(y + e_row + c));
                } else {
                    if (va) y[e_row + c] = __uint_as_float(ra.ybits);
                    if (vb) y[e_row + c + 1] = __uint_as_float(rb.ybits);
                }
                if (g.y64) {
                    if (vb && y64_pairs) *(d2 *)(g.y64 + e_row + c) = cur[u];
                    else {
                        if (va) g.y64[e_row + c] = oa;
                        if (vb) g.y64[e_row + c + 1] = ob;
                    }
                }
                const bool la = va && ra.logged, lb = vb && rb.logged;
                const uint32_t pos = j * cols + c;          // position among this wave's outputs
                if (DENSE) {
                    if (va) codes[pos] = (uint8_t)(la ? (ra.up ? 2u : 0u) : 1u);
                    if (vb) codes[pos + 1] = (uint8_t)(lb ? (rb.up ? 2u : 0u) : 1u);
                    wcount += (la ? 1u : 0u) + (lb ? 1u : 0u);
                } else {
                    const uint64_t m0 = ballot(la), m1 = ballot(lb);
                    if (m0 | m1) {                          // output order: lane-major, then the pair
                        const uint32_t q0 = wcount + rank_below(m0) + rank_below(m1);
                        if (la) ent[q0] = (uint16_t)(pos | (ra.up ? 0x8000u : 0u));
                        if (lb) ent[q0 + (la ? 1u : 0u)] = (uint16_t)((pos + 1u) | (rb.up ? 0x8000u : 0u));
                        wcount += popc64(m0) + popc64(m1);
                    }
                }
            }
        }
        if constexpr (PREFETCH) {
#pragma unroll
            for (int u = 0; u < U; ++u) cur[u] = nxt[u];
        } else {
            if (j + 1 < nrows) load_row<U>(g.a + (uint64_t)(r + 1) * cols, cols, lane, cur);
        }
    }

    if (DENSE) {
        wave_lds_fence();
        // this wave's outputs start at a multiple of five: whole bytes of the log, four per lane and pass
        const uint32_t cnt = nrows * cols, nbytes = (cnt + 4u) / 5u;
        const uint64_t byte0 = (uint64_t)group * cols;      // (r0 * cols) / 5
        const bool word_ok = ((byte0 & 3u) == 0);
        for (uint32_t b = 4u * lane; b < nbytes; b += 256u) {
            uint32_t packed = 0;
            if (5u * b + 20u <= cnt) {
                uint32_t w[5];
#pragma unroll
                for (int q = 0; q < 5; ++q) w[q] = *(const uint32_t *)(codes + 5u * b + 4u * q);
#pragma unroll
                for (int q = 0; q < 4; ++q) {               // byte q: codes 5 q .. 5 q + 4
                    uint32_t byte = 0, weight = 1;
#pragma unroll
                    for (int i = 0; i < 5; ++i) {
                        const int cc = 5 * q + i;
                        byte += ((w[cc >> 2] >> (8 * (cc & 3))) & 0xFFu) * weight;
                        weight *= 3u;
                    }
                    packed |= byte << (8 * q);
                }
            } else {                                        // the end of the wave's outputs: code 1 past it
                for (uint32_t q = 0; q < 4; ++q) {
                    uint32_t byte = 0, weight = 1;
                    for (uint32_t i = 0; i < 5; ++i) {
                        const uint32_t at = 5u * (b + q) + i;
                        byte += (at < cnt ? (uint32_t)codes[at] : 1u) * weight;
                        weight *= 3u;
                    }
                    packed |= byte << (8 * q);
                }
            }
            if (word_ok && b + 4u <= nbytes) *(uint32_t *)(tlog + byte0 + b) = packed;
            else {
                for (uint32_t q = 0; q < 4; ++q)
                    if (b + q < nbytes) tlog[byte0 + b + q] = (uint8_t)(packed >> (8 * q));
            }
        }
        if (slots) {
            const uint32_t logged = wave_sum(wcount);
            if (lane == 0 && logged)
                atomicAdd((unsigned long long *)(slots + (group % kRwSlots) * kRwSlotStride), (unsigned long long)logged);
        }
        return;
    }

    if (lane == 0) s_wc[wv] = wcount;
    __syncthreads();
    uint32_t pre[kRwWaves + 1];
    pre[0] = 0;
#pragma unroll
    for (int w = 0; w < kRwWaves; ++w) pre[w + 1] = pre[w] + s_wc[w];
    const uint32_t c = pre[kRwWaves];
    if (c == 0) {                                           // nothing to place: publish the count and go
        if (tid == 0) st_store(st + tile, kCountFlag);
        return;
    }
    // One wave trades the count for the tile's place in the log; all four then write entries (a tile
    // of twenty rows can hold thousands, and the workgroup's LDS is held until the last one has left
    // anyway, so the other waves lose nothing by waiting here).
    __shared__ uint64_t s_off;
    __shared__ uint32_t s_ok;
    if (wv == 0) {
        uint64_t off;
        const bool ok = tile_offset(st, tile, c, err, lane, off);
        if (lane == 0) { s_off = off; s_ok = ok ? 1u : 0u; }
    }
    __syncthreads();
    if (!s_ok) return;
    emit_tile_entries<kRwWaves>((const uint16_t *)smem, kWaveOut, 0x7FFFu, pre, (uint64_t)tile * kRwWaves * kRwRows * cols,
                                kRwRows * cols, s_off, cap, idx, dir, lane, wv, kRwWaves);
}

template <int OP, int U, bool DENSE>
hipError_t launch_u(const LayerArgs &g, uint32_t rows, uint32_t thr, uint32_t k, float *y, uint8_t *tlog, uint64_t *slots,
                    uint64_t *st, uint32_t tiles, uint32_t *err, const LogOut &log, hipStream_t s)
{
    const dim3 grid(tiles + (DENSE ? 0u : 1u)), block(256);
    if (k == 0)
        rowwise_kernel<OP, U, true, DENSE><<<grid, block, 0, s>>>(g, rows, thr, k, y, tlog, slots, st, tiles, err, log.idx,
                                                                  log.dir, log.cap, log.count);
    else
        rowwise_kernel<OP, U, false, DENSE><<<grid, block, 0, s>>>(g, rows, thr, k, y, tlog, slots, st, tiles, err, log.idx,
                                                                   log.dir, log.cap, log.count);
    return hipGetLastError();
}

template <int OP, bool DENSE>
hipError_t launch_op(const LayerArgs &g, uint32_t rows, uint32_t thr, uint32_t k, float *y, uint8_t *tlog, uint64_t *slots,
                     uint64_t *st, uint32_t tiles, uint32_t *err, const LogOut &log, hipStream_t s)
{
    if (g.cols <= 512) return launch_u<OP, 4, DENSE>(g, rows, thr, k, y, tlog, slots, st, tiles, err, log, s);
    if (g.cols <= 1024) return launch_u<OP, 8, DENSE>(g, rows, thr, k, y, tlog, slots, st, tiles, err, log, s);
    return hipErrorInvalidValue;
}

}  // namespace

bool rowwise_usable(int op, uint64_t cols)
{
    return (op == kLayerNorm || op == kLayerSoftmax) && cols >= kRowwiseMinCols && cols <= kRowwiseMaxCols;
}

size_t rowwise_bytes(uint64_t rows)
{
    const uint64_t tiles = (rows + kRwWaves * kRwRows - 1) / (kRwWaves * kRwRows);
    return (size_t)((tiles * 8 + 255) / 256 * 256 + 256);
}

// packed log: `slots` = dense_count_bytes() of scratch (or null when the count is not wanted)
hipError_t launch_rowwise_dense(const LayerArgs &g, uint64_t rows, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    if (rows == 0 || !n_logged) slots = nullptr;           // nothing to count, or nobody asks
    hipError_t e = launch_count_begin(slots, n_logged, s);
    if (e != hipSuccess || rows == 0) return e;
    const uint32_t tiles = (uint32_t)((rows + kRwWaves * kRwRows - 1) / (kRwWaves * kRwRows));
    const LogOut none{nullptr, nullptr, 0, nullptr};
    if (g.op == kLayerNorm)
        e = launch_op<kLayerNorm, true>(g, (uint32_t)rows, thr, k, y, tlog, slots, nullptr, tiles, nullptr, none, s);
    else
        e = launch_op<kLayerSoftmax, true>(g, (uint32_t)rows, thr, k, y, tlog, slots, nullptr, tiles, nullptr, none, s);
    if (e == hipSuccess && slots) e = launch_count_end(slots, n_logged, s);
    return e;
}

// index-list log: ws = rowwise_bytes(rows) of scratch (status words of the tiles, then the error words)
hipError_t launch_rowwise_onepass(const LayerArgs &g, uint64_t rows, uint32_t thr, uint32_t k, float *y, void *ws,
                                  const LogOut &log, hipStream_t s)
{
    const uint64_t n = rows * (uint64_t)g.cols;
    const uint32_t tiles = (uint32_t)((rows + kRwWaves * kRwRows - 1) / (kRwWaves * kRwRows));
    uint64_t *st = (uint64_t *)ws;
    uint32_t *err = (uint32_t *)((char *)ws + ((uint64_t)tiles * 8 + 255) / 256 * 256);
    hipError_t e = launch_onepass_init(st, tiles, err, log, n, s);
    if (e != hipSuccess || tiles == 0) return e;
    if (g.op == kLayerNorm)
        return launch_op<kLayerNorm, false>(g, (uint32_t)rows, thr, k, y, nullptr, nullptr, st, tiles, err, log, s);
    return launch_op<kLayerSoftmax, false>(g, (uint32_t)rows, thr, k, y, nullptr, nullptr, st, tiles, err, log, s);
}

}  // namespace vt
