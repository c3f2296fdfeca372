// vt_scan.h -- ordered offsets for tiles of one launch without a second pass: the scanner workgroup.
//
// A tile publishes the number of log entries it holds in its status word and (if it has any) waits
// until the scanner has replaced the count by the tile's offset in the globally ordered log.
// Workgroup 0 of the launch is the scanner: it polls up to 1024 consecutive status words per round,
// takes the prefix of them that is already published, scans it in LDS and writes the offsets back, so
// the log position of a tile costs two memory round trips however many tiles are in flight, and the
// scan advances by up to 1024 tiles per round trip.  Integer sums in tile order: the result does not
// depend on timing.
//
// Progress: the scanner is workgroup 0, dispatched first, and depends only on tiles publishing their
// counts, which no tile waits for anything to do; tiles depend only on the scanner.  Every wait is
// bounded all the same: after kSpinLimit polls without progress (seconds) a waiter sets the error word,
// which releases every other waiter too, so the grid always drains; a tile that gives up writes no
// entries, and the host-visible result is then *count = UINT64_MAX (VT_COUNT_ABANDONED).
// The status words and the error words must be zero when the launch starts.
#pragma once
#include "vt_device.h"

namespace vt {

namespace {

constexpr int kScannerThreads = 256, kScannerPer = 4;      // scanner: 1024 status words per round
constexpr uint32_t kSpinLimit = 1u << 21;   // polls (each a few microseconds) before a tile gives up waiting
// The scanner waits for tiles to be dispatched at all, which other work on the GPU can delay: its
// limit is longer (some tens of seconds of idle polling).
constexpr uint32_t kScanIdleLimit = 1u << 24;

constexpr uint64_t kCountFlag = 1ull << 62, kOffsetFlag = 2ull << 62, kValMask = (1ull << 62) - 1;

__device__ __forceinline__ uint64_t st_load(const uint64_t *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_store(uint64_t *p, uint64_t v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workgroup 0: turns published counts into offsets, in tile order.
__device__ __forceinline__ void scanner(uint64_t *__restrict__ st, uint32_t tiles, uint32_t *__restrict__ err,
                                        uint64_t *__restrict__ count, uint32_t *s_u32)
{
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
    uint32_t *s_min = s_u32;          // [4] first unpublished position per wave
    uint32_t *s_sum = s_u32 + 4;      // [4] count total per wave
    uint64_t run = 0;
    uint32_t base = 0, idle = 0, rounds = 0, idle_rounds = 0;
    bool force = false;
    while (base < tiles) {
        uint64_t v[kScannerPer];
        uint32_t first = kScannerPer;                        // first unpublished among my four
#pragma unroll
        for (int j = kScannerPer - 1; j >= 0; --j) {
            const uint64_t t = (uint64_t)base + tid * kScannerPer + j;
            v[j] = t < tiles ? st_load(st + t) : kCountFlag;   // past the end: published, count 0
            if (force && (v[j] >> 62) == 0) v[j] = kCountFlag;
            if ((v[j] >> 62) == 0) first = j;
        }
        uint32_t pos = first < kScannerPer ? tid * kScannerPer + first : kScannerThreads * kScannerPer;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const uint32_t other = __shfl_xor(pos, o, 64);
            pos = other < pos ? other : pos;
        }
        if (lane == 0) s_min[wv] = pos;
        __syncthreads();
        uint32_t R = s_min[0];
#pragma unroll
        for (int w = 1; w < kScannerThreads / 64; ++w) R = s_min[w] < R ? s_min[w] : R;
        if (R > tiles - base) R = tiles - base;
        ++rounds;
        if (R == 0) {                                      // nothing new yet
            ++idle_rounds;
            __syncthreads();
            if (++idle > kScanIdleLimit) {                 // never expected: stop waiting, drain
                if (tid == 0) atomicOr(err, 1u);
                force = true;
            }
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        idle = 0;
        // exclusive scan of the counts of tiles base .. base + R - 1
        uint32_t c[kScannerPer], mine = 0;
#pragma unroll
        for (int j = 0; j < kScannerPer; ++j) {
            c[j] = tid * kScannerPer + j < R ? (uint32_t)(v[j] & kValMask) : 0u;
            mine += c[j];
        }
        uint32_t incl = mine;                              // inclusive scan across the wave
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const uint32_t up = __shfl_up(incl, o, 64);
            if (lane >= (uint32_t)o) incl += up;
        }
        if (lane == 63) s_sum[wv] = incl;
        __syncthreads();
        uint32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kScannerThreads / 64; ++w) {
            if ((uint32_t)w < wv) before += s_sum[w];
            total += s_sum[w];
        }
        uint64_t off = run + before + (incl - mine);
#pragma unroll
        for (int j = 0; j < kScannerPer; ++j) {
            const uint32_t q = tid * kScannerPer + j;
            if (q < R) st_store(st + base + q, kOffsetFlag | off);
            off += c[j];
        }
        run += total;
        base += R;
        __syncthreads();                                   // s_min / s_sum are reused next round
    }
    if (tid == 0) {
        *count = __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ? ~0ull : run;
        err[1] = rounds;                                   // diagnostics: scan rounds, of which idle
        err[2] = idle_rounds;
    }
}

// A tile's side: publish the count `c` (lane 0 of the calling wave), then poll for the offset.  Returns
// false when the wait was given up (the caller writes no entries).  Called by one whole wave.
__device__ __forceinline__ bool tile_offset(uint64_t *__restrict__ st, uint32_t tile, uint32_t c, uint32_t *__restrict__ err,
                                            uint32_t lane, uint64_t &off)
{
    if (lane == 0) st_store(st + tile, kCountFlag | c);
    off = 0;
    if (c == 0) return true;                      // nothing to place: no need to wait
    for (uint32_t spins = 0;; ++spins) {
        // polls are round trips to memory and compete with the stream: a scan round takes a
        // few microseconds, so poll about that often (s_sleep 127 = 8128 cycles)
        __builtin_amdgcn_s_sleep(127);
        const uint64_t sv = st_load(st + tile);
        if ((sv >> 62) == 2) { off = sv & kValMask; return true; }
        const bool failed = __hip_atomic_load(err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0;
        if (failed || spins > kSpinLimit) {       // never expected: give up, do not hang, write no entries
            if (lane == 0) atomicOr(err, 1u);
            return false;
        }
    }
}

// Emission of a tile's entries by one wave.  The tile is WAVES chunks of `chunk_elems` consecutive
// outputs starting at output `first`; chunk w holds pre[w + 1] - pre[w] entries at ent + w * pitch, in
// output order, each the output's position in its chunk (bits 0 .. 14, under pos_mask) and its
// direction (bit 15).  The entries go to log positions off .. off + pre[WAVES] - 1 (those below `cap`),
// 256 at a time, aligned in log position: four consecutive entries per lane (one 16-byte index store
// where the log is aligned), their direction bits gathered over eight lanes into whole 32-bit words
// (the words were cleared beforehand, so partial ones are OR-ed).  Several waves may share the work:
// the calling wave takes every `parts`-th group of 256 from group `part` on.
template <int WAVES>
__device__ __forceinline__ void emit_tile_entries(const uint16_t *__restrict__ ent, uint32_t pitch, uint32_t pos_mask,
                                                  const uint32_t (&pre)[WAVES + 1], uint64_t first, uint32_t chunk_elems,
                                                  uint64_t off, uint64_t cap, uint32_t *__restrict__ idx,
                                                  uint32_t *__restrict__ dir, uint32_t lane, uint32_t part = 0,
                                                  uint32_t parts = 1)
{
    const uint32_t c = pre[WAVES];
    const uint64_t end = off + c < cap ? off + c : cap;
    const bool wide = ((uintptr_t)idx & 15u) == 0;
    for (uint64_t G = (off & ~255ull) + 256ull * part; G < end; G += 256ull * parts) {
        const uint64_t p0 = G + 4u * lane;
        uint32_t iv[4] = {0, 0, 0, 0}, nib_v = 0, nib_d = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t p = p0 + j;
            if (p >= off && p < end) {
                const uint32_t q = (uint32_t)(p - off);
                uint32_t chunk = 0, start = 0;
#pragma unroll
                for (int w = 1; w < WAVES; ++w)
                    if (q >= pre[w]) { chunk = w; start = pre[w]; }
                const uint32_t e = ent[chunk * pitch + (q - start)];
                iv[j] = (uint32_t)(first + (uint64_t)chunk * chunk_elems + (e & pos_mask));
                nib_v |= 1u << j;
                nib_d |= (e >> 15) << j;
            }
        }
        if (wide && nib_v == 0xFu) {
            typedef uint32_t u4 __attribute__((ext_vector_type(4)));
            u4 o;
            o.x = iv[0]; o.y = iv[1]; o.z = iv[2]; o.w = iv[3];
            __builtin_nontemporal_store(o, (u4 *)(idx + p0));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((nib_v >> j) & 1u) __builtin_nontemporal_store(iv[j], idx + p0 + j);
        }
        uint32_t vv = nib_v << (4u * (lane & 7u)), dv = nib_d << (4u * (lane & 7u));
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) {
            vv |= (uint32_t)__shfl_xor((int)vv, o, 64);
            dv |= (uint32_t)__shfl_xor((int)dv, o, 64);
        }
        if ((lane & 7u) == 0 && vv) {
            uint32_t *wp = dir + (G >> 5) + (lane >> 3);
            if (vv == 0xFFFFFFFFu) *wp = dv;
            else if (dv) atomicOr(wp, dv);
        }
    }
}

}  // namespace

}  // namespace vt
