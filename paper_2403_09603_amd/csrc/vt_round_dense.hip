// vt_round_dense.hip -- the log in the paper's own storage format (gfx950, wave64).
//
// One ternary entry per output (2 rounded up, 0 rounded down, 1 ignore), five entries per byte
// by radix-3 to radix-2 conversion: byte k holds elements 5k .. 5k+4, element 5k+j with weight
// 3^j; the tail of the last byte holds 1.  The format is positional, so neither side needs a
// scan or a search: both kernels are plain streams, 8 B in and 4.2 B out per element (trainer),
// 8.2 B in and 4 B out (auditor).
//
// A wavefront works on 1280 consecutive elements: ten rows of 128, each lane loading two
// neighbouring values per row (16-byte, coalesced), all ten loads in flight at once; one
// workgroup of four waves per 5120 elements, as the plain convert-copy that reaches the highest
// bandwidth on this part is shaped.  Five consecutive elements live in different lanes, so the
// codes cross the wave through LDS: written by (row, lane), read back twenty at a time by the
// lane that packs (or unpacks) four bytes of the log.
//
// The number of logged outputs is summed into 256 counters spread over as many cache lines (one
// atomic per wave; atomics on a single address would serialise at about 11 ns each, longer than
// the whole stream) and folded by a one-workgroup kernel afterwards.
#include "vt_device.h"
#include "vt_kernels.h"
#include "vt_source.h"

#include <type_traits>

namespace vt {

namespace {

typedef double d2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

constexpr int kRows = 10;                     // rows of 128 per wave: 1280 elements, 256 log bytes
constexpr uint32_t kChunk = 128u * kRows;
constexpr int kWaves = 4;                     // 256 threads
constexpr uint32_t kTile = kChunk * kWaves;   // 5120 elements, 1024 log bytes per workgroup
constexpr uint32_t kSlots = 256, kSlotStride = 8;   // counters, one per 64-byte line (in uint64 units)

__global__ __launch_bounds__(256) void zero_slots_kernel(uint64_t *slots) { slots[threadIdx.x * kSlotStride] = 0; }

__global__ __launch_bounds__(256) void sum_slots_kernel(const uint64_t *__restrict__ slots, uint64_t *__restrict__ out)
{
    __shared__ unsigned long long total;
    if (threadIdx.x == 0) total = 0;
    __syncthreads();
    atomicAdd(&total, (unsigned long long)slots[threadIdx.x * kSlotStride]);     // integer sum: order-free
    __syncthreads();
    if (threadIdx.x == 0) *out = total;
}

__global__ void zero_u64_kernel(uint64_t *p) { *p = 0; }

// Consecutive workgroup ids run on different XCDs; every XCD takes one contiguous eighth of the tiles.
__device__ __forceinline__ uint32_t xcd_contiguous_tile()
{
    const uint32_t i = blockIdx.x, q = gridDim.x / 8u, r = gridDim.x % 8u, xcd = i % 8u;
    return xcd * q + (xcd < r ? xcd : r) + i / 8u;
}

// ternary code and FP32 bits of one value
template <bool K0>
__device__ __forceinline__ uint32_t code_of(double x, uint32_t thr, uint32_t k, uint32_t &ybits)
{
    const Rounded r = round_decide<K0>(x, thr, k);
    ybits = r.ybits;
    return r.logged ? (r.up ? 2u : 0u) : 1u;
}

template <bool FULL, bool VEC, class Src>
__device__ __forceinline__ void load_rows(const Src &src, uint64_t n, uint64_t base, uint32_t lane, d2 (&v)[kRows])
{
#pragma unroll
    for (int u = 0; u < kRows; ++u)                               // past the end: 1.0, never logged (code 1 in the tail)
        v[u] = src.template pair<FULL, VEC>(base + (uint64_t)u * 128u + 2u * lane, n);
#pragma unroll
    for (int u = 0; u < kRows; ++u) src.template keep<FULL, VEC>(base + (uint64_t)u * 128u + 2u * lane, n, v[u]);
}

template <bool FULL, bool VEC>
__device__ __forceinline__ void store_pair(float *__restrict__ y, uint64_t n, uint64_t e, uint32_t ya, uint32_t yb)
{
    if (VEC && (FULL || e + 1 < n)) {
        f2 o;
        o.x = __uint_as_float(ya);
        o.y = __uint_as_float(yb);
        __builtin_nontemporal_store(o, (f2 *)(y + e));
    } else {
        if (e < n) y[e] = __uint_as_float(ya);
        if (e + 1 < n) y[e + 1] = __uint_as_float(yb);
    }
}

// Trainer: y = rnd_32(x), tlog = packed codes.  One workgroup per 5120 elements.
template <bool FULL, bool VEC, bool K0, class Src>
__device__ __forceinline__ void round_log_dense_chunk(const Src &x, uint64_t n, uint32_t thr, uint32_t k,
                                                      float *__restrict__ y, uint8_t *__restrict__ tlog,
                                                      uint64_t base, uint32_t lane, uint8_t *__restrict__ mine,
                                                      uint64_t *__restrict__ slots)
{
    d2 v[kRows];
    load_rows<FULL, VEC>(x, n, base, lane, v);
    uint32_t logged = 0;
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        uint32_t ya, yb;
        const uint32_t ca = code_of<K0>(v[u].x, thr, k, ya), cb = code_of<K0>(v[u].y, thr, k, yb);
        store_pair<FULL, VEC>(y, n, base + (uint64_t)u * 128u + 2u * lane, ya, yb);
        logged += (ca != 1u) + (cb != 1u);
        *(uint16_t *)(mine + u * 128 + 2 * lane) = (uint16_t)(ca | (cb << 8));
    }
    wave_lds_fence();
    // this lane packs elements 20 lane .. 20 lane + 19 of the chunk: four bytes of the log
    uint32_t w[5];
#pragma unroll
    for (int k = 0; k < 5; ++k) w[k] = *(const uint32_t *)(mine + 20 * lane + 4 * k);
    uint32_t packed = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {                                 // byte q: codes 5 q .. 5 q + 4
        uint32_t byte = 0, weight = 1;
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int c = 5 * q + j;
            byte += ((w[c >> 2] >> (8 * (c & 3))) & 0xFFu) * weight;
            weight *= 3u;
        }
        packed |= byte << (8 * q);
    }
    const uint64_t byte0 = base / 5u + 4u * lane;                 // base is a multiple of 1280
    if (FULL) *(uint32_t *)(tlog + byte0) = packed;
    else {
        const uint64_t nbytes = (n + 4) / 5;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (byte0 + q < nbytes) tlog[byte0 + q] = (uint8_t)(packed >> (8 * q));
    }
    if (slots) {
        logged = wave_sum(logged);
        if (lane == 0 && logged)
            atomicAdd((unsigned long long *)(slots + ((blockIdx.x * kWaves + (threadIdx.x >> 6)) % kSlots) * kSlotStride),
                      (unsigned long long)logged);
    }
}

template <bool VEC, bool K0, class Src>
__global__ __launch_bounds__(kWaves * 64) void round_log_dense_kernel(const Src x, uint64_t n, uint32_t thr,
                                                              uint32_t k, float *__restrict__ y,
                                                              uint8_t *__restrict__ tlog, uint64_t *__restrict__ slots)
{
    __shared__ __attribute__((aligned(16))) uint8_t codes[kWaves][kChunk];
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const uint64_t base = (uint64_t)xcd_contiguous_tile() * kTile + (uint64_t)wv * kChunk;
    if (base >= n) return;
    if (base + kChunk <= n) round_log_dense_chunk<true, VEC, K0>(x, n, thr, k, y, tlog, base, lane, codes[wv], slots);
    else round_log_dense_chunk<false, VEC, K0>(x, n, thr, k, y, tlog, base, lane, codes[wv], slots);
}

// Auditor: entry i of the packed log applied to x[i].
template <bool FULL, bool VEC, bool K0>
__device__ __forceinline__ void replay_dense_chunk(const double *__restrict__ x, uint64_t n,
                                                   const uint8_t *__restrict__ tlog, float *__restrict__ y,
                                                   uint64_t base, uint32_t lane, uint8_t *__restrict__ mine, uint32_t k)
{
    d2 v[kRows];
    load_rows<FULL, VEC>(PlainSource{x}, n, base, lane, v);
    // four bytes of the log -> twenty codes, written where their elements' lanes will look
    const uint64_t byte0 = base / 5u + 4u * lane;
    uint32_t packed = 0x79797979u;                                // 0x79 = 121 = five times "ignore"
    if (FULL) packed = *(const uint32_t *)(tlog + byte0);
    else {
        const uint64_t nbytes = (n + 4) / 5;
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (byte0 + q < nbytes) packed = (packed & ~(0xFFu << (8 * q))) | ((uint32_t)tlog[byte0 + q] << (8 * q));
    }
    uint32_t w[5] = {0, 0, 0, 0, 0};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        uint32_t byte = (packed >> (8 * q)) & 0xFFu;
#pragma unroll
        for (int j = 0; j < 5; ++j) {
            const int c = 5 * q + j;
            w[c >> 2] |= (byte % 3u) << (8 * (c & 3));
            byte /= 3u;
        }
    }
#pragma unroll
    for (int k = 0; k < 5; ++k) *(uint32_t *)(mine + 20 * lane + 4 * k) = w[k];
    wave_lds_fence();
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
        const uint32_t cw = *(const uint16_t *)(mine + u * 128 + 2 * lane);
        const uint32_t ca = cw & 0xFFu, cb = cw >> 8;
        const uint64_t ba = (uint64_t)__double_as_longlong(v[u].x), bb = (uint64_t)__double_as_longlong(v[u].y);
        // unlogged: nearest (hardware conversion where it cannot differ from the definition);
        // logged: toward the recorded side
        uint32_t ya, yb;
        if (K0) {
            const FastDecision fa = decide_fast(v[u].x), fb = decide_fast(v[u].y);
            ya = __float_as_uint(fa.y);
            yb = __float_as_uint(fb.y);
            if (__builtin_expect(fa.slow, 0)) { if (v[u].x != 0.0) ya = decide(ba).ybits; }   // (+-0: the conversion stands)
            if (__builtin_expect(fb.slow, 0)) { if (v[u].y != 0.0) yb = decide(bb).ybits; }
            if (ca != 1u) ya = directed(ba, ca >> 1);
            if (cb != 1u) yb = directed(bb, cb >> 1);
        } else {
            ya = ca != 1u ? directed_k(ba, ca >> 1, k) : decide_k(ba, k).ybits;
            yb = cb != 1u ? directed_k(bb, cb >> 1, k) : decide_k(bb, k).ybits;
        }
        store_pair<FULL, VEC>(y, n, base + (uint64_t)u * 128u + 2u * lane, ya, yb);
    }
}

template <bool VEC, bool K0>
__global__ __launch_bounds__(kWaves * 64) void replay_dense_kernel(const double *__restrict__ x, uint64_t n,
                                                           const uint8_t *__restrict__ tlog, float *__restrict__ y,
                                                           uint32_t k)
{
    __shared__ __attribute__((aligned(16))) uint8_t codes[kWaves][kChunk];
    const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
    const uint64_t base = (uint64_t)xcd_contiguous_tile() * kTile + (uint64_t)wv * kChunk;
    if (base >= n) return;
    if (base + kChunk <= n) replay_dense_chunk<true, VEC, K0>(x, n, tlog, y, base, lane, codes[wv], k);
    else replay_dense_chunk<false, VEC, K0>(x, n, tlog, y, base, lane, codes[wv], k);
}

// `nbits` (1..20) plane bits of one row from column `col` on, from at most two words per plane
// (col + nbits <= ncols, so a second word lies in the same row).
__device__ __forceinline__ void plane_field(const uint64_t *__restrict__ logged, const uint64_t *__restrict__ dir,
                                            uint64_t row, uint32_t wpr, uint32_t col, uint32_t nbits, uint32_t &lg, uint32_t &up)
{
    const uint64_t w = row * wpr + (col >> 6);
    const uint32_t sh = col & 63u;
    uint64_t wl = logged[w] >> sh, wd = dir[w] >> sh;
    if (sh + nbits > 64u) {
        wl |= logged[w + 1] << (64u - sh);
        wd |= dir[w + 1] << (64u - sh);
    }
    lg = (uint32_t)wl & ((1u << nbits) - 1u);
    up = (uint32_t)wd & lg;
}

// Decision bit-planes of a dense (rows x ncols) output -> packed ternary log.  One thread per four
// bytes (twenty outputs, one 32-bit store).  The twenty plane bits are cut out as fields (two when
// the window runs over a row end: every wave has such a thread unless 20 divides ncols, so that
// case must not take a slow path), and a byte is 121 + 2 T[up bits] - T[logged bits] with
// T[b] = sum of 3^j over the set bits of b (32 entries in LDS): code 1 everywhere, minus 3^j where
// logged (code 0), plus 2 * 3^j where logged and up.  Rows shorter than twenty outputs and the end
// of the log walk bit by bit.  total < 2^32.  The workgroup's number of logged outputs goes to
// partial[blockIdx.x] (summed by count_partials_kernel: integer, any order).
__global__ __launch_bounds__(256) void planes_to_dense_kernel(const uint64_t *__restrict__ logged,
                                                              const uint64_t *__restrict__ dir, uint32_t wpr,
                                                              uint32_t ncols, double inv_ncols, uint64_t total,
                                                              uint8_t *__restrict__ tlog, uint32_t *__restrict__ partial)
{
    __shared__ uint32_t wave_cnt[4];
    __shared__ uint8_t T[32];
    if (threadIdx.x < 32) {
        const uint32_t b = threadIdx.x;
        T[b] = (uint8_t)((b & 1u) + 3u * ((b >> 1) & 1u) + 9u * ((b >> 2) & 1u) + 27u * ((b >> 3) & 1u) + 81u * ((b >> 4) & 1u));
    }
    __syncthreads();
    const uint64_t q = (uint64_t)blockIdx.x * 256u + threadIdx.x;       // 32-bit word of the log
    const uint64_t e0 = q * 20u;
    uint32_t n_logged = 0;
    if (e0 < total) {
        uint32_t row, col;
        divmod_u32((uint32_t)e0, ncols, inv_ncols, row, col);
        uint32_t word = 0;
        if (e0 + 20u <= total && ncols >= 20u) {
            const uint32_t n1 = ncols - col < 20u ? ncols - col : 20u;
            uint32_t lg, up;
            plane_field(logged, dir, row, wpr, col, n1, lg, up);
            if (n1 < 20u) {                                   // the rest starts the next row
                uint32_t lg2, up2;
                plane_field(logged, dir, (uint64_t)row + 1u, wpr, 0u, 20u - n1, lg2, up2);
                lg |= lg2 << n1;
                up |= up2 << n1;
            }
            n_logged = (uint32_t)__popc(lg);
#pragma unroll
            for (int by = 0; by < 4; ++by) {
                const uint32_t byte = 121u + 2u * T[(up >> (5 * by)) & 31u] - T[(lg >> (5 * by)) & 31u];
                word |= byte << (8 * by);
            }
        } else {
            uint64_t wl = 0, wd = 0;
            bool have = false;
#pragma unroll 1
            for (int by = 0; by < 4; ++by) {
                uint32_t byte = 0, weight = 1;
#pragma unroll 1
                for (int j = 0; j < 5; ++j) {
                    uint32_t code = 1;
                    if (e0 + (uint64_t)(5 * by + j) < total) {
                        if (!have) {
                            const uint64_t w = (uint64_t)row * wpr + (col >> 6);
                            wl = logged[w];
                            wd = dir[w];
                            have = true;
                        }
                        const uint32_t lg = (uint32_t)(wl >> (col & 63u)) & 1u, up = (uint32_t)(wd >> (col & 63u)) & 1u;
                        code = lg ? 2u * up : 1u;
                        n_logged += lg;
                        ++col;
                        if ((col & 63u) == 0) have = false;
                        if (col == ncols) { col = 0; ++row; have = false; }
                    }
                    byte += code * weight;
                    weight *= 3u;
                }
                word |= byte << (8 * by);
            }
        }
        const uint64_t nbytes = (total + 4) / 5;
        if (4 * q + 4 <= nbytes) {
            *(uint32_t *)(tlog + 4 * q) = word;
        } else {                                          // the log ends inside this word
            for (uint64_t i = 4 * q; i < nbytes; ++i) tlog[i] = (uint8_t)(word >> (8 * (i - 4 * q)));
        }
    }
    n_logged = wave_sum(n_logged);
    if ((threadIdx.x & 63u) == 0) wave_cnt[threadIdx.x >> 6] = n_logged;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = wave_cnt[0] + wave_cnt[1] + wave_cnt[2] + wave_cnt[3];
}

__global__ __launch_bounds__(1024) void count_partials_kernel(const uint32_t *__restrict__ partial, uint32_t n,
                                                              uint64_t *__restrict__ count)
{
    __shared__ uint64_t part[16];
    uint64_t sum = 0;
    for (uint32_t i = threadIdx.x; i < n; i += 1024u) sum += partial[i];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += (uint64_t)__shfl_xor((unsigned long long)sum, o, 64);
    if ((threadIdx.x & 63u) == 0) part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        uint64_t total = 0;
        for (int i = 0; i < 16; ++i) total += part[i];
        *count = total;
    }
}

}  // namespace

size_t dense_count_bytes() { return (size_t)kSlots * kSlotStride * 8; }

hipError_t launch_count_begin(uint64_t *slots, uint64_t *n_logged, hipStream_t s)
{
    if (slots) zero_slots_kernel<<<1, kSlots, 0, s>>>(slots);
    else if (n_logged) zero_u64_kernel<<<1, 1, 0, s>>>(n_logged);
    return hipGetLastError();
}

hipError_t launch_count_end(const uint64_t *slots, uint64_t *n_logged, hipStream_t s)
{
    sum_slots_kernel<<<1, kSlots, 0, s>>>(slots, n_logged);
    return hipGetLastError();
}

namespace {

// `slots`: dense_count_bytes() of scratch, needed when n_logged is wanted
template <class Src>
hipError_t launch_dense_from(const Src &src, bool vec, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                             uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    if (n == 0 || !n_logged) slots = nullptr;              // nothing to count, or nobody asks
    const hipError_t e0 = launch_count_begin(slots, n_logged, s);
    if (e0 != hipSuccess || n == 0) return e0;
    const uint64_t blocks = (n + kTile - 1) / kTile;
    const dim3 grid((uint32_t)blocks), block(kWaves * 64);
    if (vec && k == 0) round_log_dense_kernel<true, true, Src><<<grid, block, 0, s>>>(src, n, thr, k, y, tlog, slots);
    else if (vec) round_log_dense_kernel<true, false, Src><<<grid, block, 0, s>>>(src, n, thr, k, y, tlog, slots);
    else if constexpr (std::is_same<Src, PlainSource>::value) {     // misaligned tensors: scalar accesses
        if (k == 0) round_log_dense_kernel<false, true, Src><<<grid, block, 0, s>>>(src, n, thr, k, y, tlog, slots);
        else round_log_dense_kernel<false, false, Src><<<grid, block, 0, s>>>(src, n, thr, k, y, tlog, slots);
    } else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && slots) e = launch_count_end(slots, n_logged, s);
    return e;
}

}  // namespace

hipError_t launch_round_log_dense(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    const bool vec = ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 8 == 0);
    return launch_dense_from(PlainSource{x}, vec, n, thr, k, y, tlog, n_logged, slots, s);
}

hipError_t launch_splitk_log_dense(const SplitKArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                   uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    const SplitKSource src{a.partial, a.slab, a.splits, a.variant, a.alpha, a.bias, a.ncols ? a.ncols : 1u,
                           1.0 / (double)(a.ncols ? a.ncols : 1u), a.y64};
    return launch_dense_from(src, true, n, thr, k, y, tlog, n_logged, slots, s);
}

hipError_t launch_phase_log_dense(const PhaseArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    if (a.sh < 1 || a.sh > 2 || a.sw < 1 || a.sw > 2 || a.C == 0 || a.C % 2 || a.H == 0 || a.W == 0) return hipErrorInvalidValue;
    PhaseSource src;
    src.P = a.P; src.C = a.C; src.W = a.W; src.HW = a.H * a.W;
    src.inv_C = 1.0 / (double)a.C; src.inv_W = 1.0 / (double)a.W; src.inv_HW = 1.0 / (double)(a.H * a.W);
    src.ph = a.ph; src.pw = a.pw; src.shift_h = a.sh - 1u; src.shift_w = a.sw - 1u;
    for (int i = 0; i < 2; ++i) { src.q0h[i] = a.q0h[i]; src.Ha[i] = a.Ha[i]; src.q0w[i] = a.q0w[i]; src.Wb[i] = a.Wb[i]; }
    for (int i = 0; i < 4; ++i) src.off[i] = a.off[i];
    src.has = a.has; src.y64 = a.y64;
    return launch_dense_from(src, true, n, thr, k, y, tlog, n_logged, slots, s);
}

// the same stream with a layer evaluated on the fly as its source (inputs 16-byte aligned)
hipError_t launch_layer_log_dense(const LayerArgs &g, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s)
{
    switch (g.op) {                                              // one specialised kernel per layer
    case kLayerAdd: return launch_dense_from(LayerSource<kLayerAdd>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerRelu: return launch_dense_from(LayerSource<kLayerRelu>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerGeluTanh: return launch_dense_from(LayerSource<kLayerGeluTanh>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerGeluErf: return launch_dense_from(LayerSource<kLayerGeluErf>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerNorm: return launch_dense_from(LayerSource<kLayerNorm>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerSoftmax: return launch_dense_from(LayerSource<kLayerSoftmax>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerBatchNorm: return launch_dense_from(LayerSource<kLayerBatchNorm>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    case kLayerBatchNormRelu: return launch_dense_from(LayerSource<kLayerBatchNormRelu>{g}, true, n, thr, k, y, tlog, n_logged, slots, s);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, uint32_t k, float *y, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kTile - 1) / kTile;
    const bool vec = ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 8 == 0);
    const dim3 grid((uint32_t)blocks), block(kWaves * 64);
    if (vec && k == 0) replay_dense_kernel<true, true><<<grid, block, 0, s>>>(x, n, tlog, y, k);
    else if (vec) replay_dense_kernel<true, false><<<grid, block, 0, s>>>(x, n, tlog, y, k);
    else if (k == 0) replay_dense_kernel<false, true><<<grid, block, 0, s>>>(x, n, tlog, y, k);
    else replay_dense_kernel<false, false><<<grid, block, 0, s>>>(x, n, tlog, y, k);
    return hipGetLastError();
}

// also writes *count; uses pl.seg_cnt as scratch (one entry per workgroup of 5120 outputs: never
// more than the plane has segments of 4096)
hipError_t launch_planes_to_dense(const Planes &pl, uint64_t rows, uint8_t *tlog, uint64_t *count, hipStream_t s)
{
    const uint64_t total = rows * (uint64_t)pl.ncols;
    const uint64_t words = (total + 19) / 20;
    const uint32_t blocks = (uint32_t)((words + 255) / 256);
    if (blocks)
        planes_to_dense_kernel<<<blocks, 256, 0, s>>>(pl.logged, pl.dir, pl.wpr, pl.ncols, 1.0 / (double)(pl.ncols ? pl.ncols : 1u),
                                                      total, tlog, pl.seg_cnt);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    count_partials_kernel<<<1, 1024, 0, s>>>(pl.seg_cnt, blocks, count);
    return hipGetLastError();
}

}  // namespace vt
