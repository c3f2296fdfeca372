// vt_round_onepass.hip -- the standalone trainer hook as ONE streaming pass (gfx950, wave64).
//
// Each tile workgroup of four waves rounds 4096 FP64 values (16-byte loads, eight in flight per lane,
// non-temporal both ways: the launch shape in which a plain FP64 -> FP32 convert-copy streams fastest
// on this part; eight-wave workgroups over 8192 values measured 9 % slower for the copy alone),
// decides which outputs are logged and compacts their entries in LDS.
// The input is read once and nothing but the outputs is written, so the kernel moves exactly
// the algorithmic bytes: 8 B + 4 B per element plus 4.125 B per logged entry.
//
// Position in the globally ordered log, without a second pass over the data: workgroup 0 is a
// scanner and every tile trades its count for its offset (vt_scan.h).  Only one wave of a tile
// waits; the other three retire at once.  (Measured alternatives on 2^28 values, which stream in
// 0.50 ms: tile-to-tile decoupled look-back 0.71 ms -- its frontier moves slower than HBM retires
// tiles; per-bucket atomic totals read by every tile 2.7 ms -- polling of shared lines serialises
// at the memory side.)
#include "vt_device.h"
#include "vt_kernels.h"
#include "vt_scan.h"
#include "vt_source.h"

namespace vt {

namespace {

typedef double d2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;        // 4 waves
constexpr int kWaves = kThreads / 64;
constexpr int kWaveChunk = 1024;     // contiguous outputs per wave: 8 rows of 128
constexpr int kRows = 8;
constexpr int kTile = kWaves * kWaveChunk;   // outputs per workgroup

__global__ __launch_bounds__(256) void onepass_init_kernel(uint64_t *__restrict__ st, uint32_t tiles,
                                                           uint32_t *__restrict__ err, uint32_t *__restrict__ dir,
                                                           uint64_t dir_words, uint64_t *__restrict__ count)
{
    const uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t k = i; k < tiles; k += stride) st[k] = 0;
    for (uint64_t k = i; k < dir_words; k += stride) dir[k] = 0;
    if (i == 0) { *err = 0; if (tiles == 0) *count = 0; }
}

// One wave's share of a tile: 1024 contiguous values as 8 rows of 128 (two per lane).  FULL:
// the whole tile lies inside the array, so no access is guarded.  Returns the wave's count;
// entries go to `ent` in element order.
template <bool FULL, bool K0, class Src>
__device__ __forceinline__ uint32_t round_rows(const Src &x, uint64_t n, uint32_t thr, uint32_t k,
                                               float *__restrict__ y, uint64_t wbase, uint32_t lane,
                                               uint16_t *__restrict__ ent)
{
    d2 v[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const uint64_t e = wbase + (uint64_t)u * 128u + 2u * lane;
        v[u] = x.template pair<FULL, true>(e, n);                     // past the end: 1.0, never logged
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u) x.template keep<FULL, true>(wbase + (uint64_t)u * 128u + 2u * lane, n, v[u]);
    uint32_t wcount = 0;
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const uint64_t e = wbase + (uint64_t)u * 128u + 2u * lane;
        uint32_t ya, yb;
        bool la, lb, da, db;
        if (K0) {
            const FastDecision a = decide_fast(v[u].x), b = decide_fast(v[u].y);
            ya = __float_as_uint(a.y); yb = __float_as_uint(b.y);
            la = a.D < thr; lb = b.D < thr;
            da = a.grow != a.neg; db = b.grow != b.neg;
            if (__builtin_expect(ballot(a.slow || b.slow) != 0, 0)) {      // rare values: redo those lanes
                if (a.slow && v[u].x != 0.0) {                            // (+-0: the fast result stands)
                    const Decision d = decide((uint64_t)__double_as_longlong(v[u].x));
                    ya = d.ybits; la = d.D < thr; da = d.dir != 0;
                }
                if (b.slow && v[u].y != 0.0) {
                    const Decision d = decide((uint64_t)__double_as_longlong(v[u].y));
                    yb = d.ybits; lb = d.D < thr; db = d.dir != 0;
                }
            }
        } else {                                                           // rounding amount below 32
            const Decision a = decide_k((uint64_t)__double_as_longlong(v[u].x), k);
            const Decision b = decide_k((uint64_t)__double_as_longlong(v[u].y), k);
            ya = a.ybits; yb = b.ybits;
            la = a.D < thr; lb = b.D < thr;
            da = a.dir != 0; db = b.dir != 0;
        }
        if (FULL || e + 1 < n) {
            f2 o;
            o.x = __uint_as_float(ya);
            o.y = __uint_as_float(yb);
            __builtin_nontemporal_store(o, (f2 *)(y + e));
        } else if (e < n) {
            y[e] = __uint_as_float(ya);
        }
        if (!FULL) { la = la && e < n; lb = lb && e + 1 < n; }
        const uint64_t m0 = ballot(la), m1 = ballot(lb);
        if (m0 | m1) {
            const uint32_t r0 = wcount + rank_below(m0) + rank_below(m1);
            const uint32_t pos = (uint32_t)u * 128u + 2u * lane;
            if (la) ent[r0] = (uint16_t)(pos | (da ? 0x8000u : 0u));
            if (lb) ent[r0 + (la ? 1u : 0u)] = (uint16_t)((pos + 1u) | (db ? 0x8000u : 0u));
            wcount += popc64(m0) + popc64(m1);
        }
    }
    return wcount;
}

template <bool K0, class Src>
__global__ __launch_bounds__(kThreads) void round_log_onepass_kernel(const Src x, uint64_t n,
                                                                uint32_t thr, uint32_t k, float *__restrict__ y,
                                                                uint64_t *__restrict__ st, uint32_t tiles,
                                                                uint32_t *__restrict__ err,
                                                                uint32_t *__restrict__ idx, uint32_t *__restrict__ dir,
                                                                uint64_t cap, uint64_t *__restrict__ count)
{
    __shared__ uint16_t ent[kWaves][kWaveChunk];  // per wave: position in its chunk | direction << 15
    __shared__ uint32_t s_wc[kWaves < 8 ? 8 : kWaves];   // logged outputs per wave (scanner: its 8 words of scratch)
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
    if (blockIdx.x == 0) {
        if (tid < kScannerThreads) scanner(st, tiles, err, count, s_wc);
        return;
    }
    const uint32_t tile = blockIdx.x - 1;
    const uint64_t wbase = (uint64_t)tile * kTile + (uint64_t)wv * kWaveChunk;
    const uint32_t wcount = ((uint64_t)(tile + 1) * kTile <= n)
                                ? round_rows<true, K0>(x, n, thr, k, y, wbase, lane, ent[wv])
                                : round_rows<false, K0>(x, n, thr, k, y, wbase, lane, ent[wv]);
    if (lane == 0) s_wc[wv] = wcount;
    __syncthreads();
    // Only wave 0 goes on: it alone waits for the tile's place in the log, so the other three
    // waves free their slots for the next tiles' loads meanwhile.
    if (wv != 0) return;
    uint32_t pre[kWaves + 1];                     // exclusive prefix of the waves' counts
    pre[0] = 0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) pre[w + 1] = pre[w] + s_wc[w];
    const uint32_t c = pre[kWaves];
    uint64_t off;
    if (!tile_offset(st, tile, c, err, lane, off) || c == 0) return;
    emit_tile_entries<kWaves>(&ent[0][0], kWaveChunk, 0x3FFu, pre, (uint64_t)tile * kTile, kWaveChunk, off, cap, idx, dir, lane);
}

// Round only (threshold 0: nothing can be logged, the count is 0).  No scan, no status words: the
// plain FP64 -> FP32 stream in the launch shape that measured fastest on this part -- workgroups of
// four waves over 1024 values (two rows of 128 per wave), every XCD taking runs of 64 consecutive
// workgroups inside one moving window of 512 -- 6.4 to 6.6 TB/s on 2^28 values, the practical ceiling
// the other streaming kernels are held against.
constexpr int kRoTile = 1024;
template <bool K0>
__global__ __launch_bounds__(256) void round_only_kernel(const double *__restrict__ x, uint64_t n, uint32_t k,
                                                         float *__restrict__ y, uint64_t *__restrict__ count)
{
    const uint32_t i = blockIdx.x, window = i / 512u;
    const uint32_t tile = (window + 1u) * 512u <= gridDim.x ? window * 512u + (i % 8u) * 64u + (i / 8u) % 64u : i;
    if (i == 0 && threadIdx.x == 0) *count = 0;
    const uint64_t base = (uint64_t)tile * kRoTile + (uint64_t)(threadIdx.x >> 6) * 256u + 2u * (threadIdx.x & 63u);
    const bool full = (uint64_t)(tile + 1u) * kRoTile <= n;
    const PlainSource src{x};
    d2 v[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) v[u] = full ? src.pair<true, true>(base + 128u * u, n) : src.pair<false, true>(base + 128u * u, n);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const uint64_t e = base + 128u * u;
        const Rounded a = round_decide<K0>(v[u].x, 0u, k), b = round_decide<K0>(v[u].y, 0u, k);
        if (full || e + 1 < n) {
            f2 o;
            o.x = __uint_as_float(a.ybits);
            o.y = __uint_as_float(b.ybits);
            __builtin_nontemporal_store(o, (f2 *)(y + e));
        } else if (e < n) {
            y[e] = __uint_as_float(a.ybits);
        }
    }
}

}  // namespace

// y = rnd(x) and *count = 0 (x 16-byte, y 8-byte aligned, as for the single-pass kernel; n > 0)
hipError_t launch_round_only(const double *x, uint64_t n, uint32_t k, float *y, uint64_t *count, hipStream_t s)
{
    const uint32_t tiles = (uint32_t)((n + kRoTile - 1) / kRoTile);
    if (k == 0) round_only_kernel<true><<<tiles, 256, 0, s>>>(x, n, k, y, count);
    else round_only_kernel<false><<<tiles, 256, 0, s>>>(x, n, k, y, count);
    return hipGetLastError();
}

size_t onepass_bytes(uint64_t n)
{
    const uint64_t tiles = (n + kTile - 1) / kTile;
    return (size_t)((tiles * 8 + 255) / 256 * 256 + 256);
}

bool onepass_usable(const double *x, const float *y)
{
    return ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 8 == 0);
}

// zeroes the status words of `tiles` tiles, the error words, the direction words that n outputs can
// fill, and (when there are no tiles) the count
hipError_t launch_onepass_init(uint64_t *st, uint32_t tiles, uint32_t *err, const LogOut &log, uint64_t n, hipStream_t s)
{
    const uint64_t stored = log.cap < n ? log.cap : n;
    const uint64_t dir_words = (stored + 31) / 32;
    const uint64_t work = tiles > dir_words ? tiles : dir_words;
    uint32_t blocks = (uint32_t)((work + 1023) / 1024);
    if (blocks < 1) blocks = 1;
    if (blocks > 4096) blocks = 4096;
    onepass_init_kernel<<<blocks, 256, 0, s>>>(st, tiles, err, log.dir, dir_words, log.count);
    return hipGetLastError();
}

namespace {

template <class Src>
hipError_t launch_onepass_from(const Src &src, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                               const LogOut &log, hipStream_t s)
{
    const uint32_t tiles = (uint32_t)((n + kTile - 1) / kTile);
    uint64_t *st = (uint64_t *)ws;
    uint32_t *err = (uint32_t *)((char *)ws + ((uint64_t)tiles * 8 + 255) / 256 * 256);
    hipError_t e = launch_onepass_init(st, tiles, err, log, n, s);
    if (e != hipSuccess || tiles == 0) return e;
    if (k == 0)
        round_log_onepass_kernel<true, Src><<<tiles + 1, kThreads, 0, s>>>(src, n, thr, k, y, st, tiles, err, log.idx,
                                                                           log.dir, log.cap, log.count);
    else
        round_log_onepass_kernel<false, Src><<<tiles + 1, kThreads, 0, s>>>(src, n, thr, k, y, st, tiles, err, log.idx,
                                                                            log.dir, log.cap, log.count);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_round_log_onepass(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s)
{
    return launch_onepass_from(PlainSource{x}, n, thr, k, y, ws, log, s);
}

// the same pass with a layer evaluated on the fly as its source (inputs 16-byte, y 8-byte aligned)
hipError_t launch_splitk_log_onepass(const SplitKArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                     const LogOut &log, hipStream_t s)
{
    const SplitKSource src{a.partial, a.slab, a.splits, a.variant, a.alpha, a.bias, a.ncols ? a.ncols : 1u,
                           1.0 / (double)(a.ncols ? a.ncols : 1u), a.y64};
    return launch_onepass_from(src, n, thr, k, y, ws, log, s);
}

hipError_t launch_phase_log_onepass(const PhaseArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s)
{
    if (a.sh < 1 || a.sh > 2 || a.sw < 1 || a.sw > 2 || a.C == 0 || a.C % 2 || a.H == 0 || a.W == 0) return hipErrorInvalidValue;
    PhaseSource src;
    src.P = a.P; src.C = a.C; src.W = a.W; src.HW = a.H * a.W;
    src.inv_C = 1.0 / (double)a.C; src.inv_W = 1.0 / (double)a.W; src.inv_HW = 1.0 / (double)(a.H * a.W);
    src.ph = a.ph; src.pw = a.pw; src.shift_h = a.sh - 1u; src.shift_w = a.sw - 1u;
    for (int i = 0; i < 2; ++i) { src.q0h[i] = a.q0h[i]; src.Ha[i] = a.Ha[i]; src.q0w[i] = a.q0w[i]; src.Wb[i] = a.Wb[i]; }
    for (int i = 0; i < 4; ++i) src.off[i] = a.off[i];
    src.has = a.has; src.y64 = a.y64;
    return launch_onepass_from(src, n, thr, k, y, ws, log, s);
}

hipError_t launch_layer_log_onepass(const LayerArgs &g, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s)
{
    switch (g.op) {                                              // one specialised kernel per layer
    case kLayerAdd: return launch_onepass_from(LayerSource<kLayerAdd>{g}, n, thr, k, y, ws, log, s);
    case kLayerRelu: return launch_onepass_from(LayerSource<kLayerRelu>{g}, n, thr, k, y, ws, log, s);
    case kLayerGeluTanh: return launch_onepass_from(LayerSource<kLayerGeluTanh>{g}, n, thr, k, y, ws, log, s);
    case kLayerGeluErf: return launch_onepass_from(LayerSource<kLayerGeluErf>{g}, n, thr, k, y, ws, log, s);
    case kLayerNorm: return launch_onepass_from(LayerSource<kLayerNorm>{g}, n, thr, k, y, ws, log, s);
    case kLayerSoftmax: return launch_onepass_from(LayerSource<kLayerSoftmax>{g}, n, thr, k, y, ws, log, s);
    case kLayerBatchNorm: return launch_onepass_from(LayerSource<kLayerBatchNorm>{g}, n, thr, k, y, ws, log, s);
    case kLayerBatchNormRelu: return launch_onepass_from(LayerSource<kLayerBatchNormRelu>{g}, n, thr, k, y, ws, log, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace vt
