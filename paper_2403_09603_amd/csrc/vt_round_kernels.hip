// vt_round_kernels.hip -- HBM-bound kernels of the trainer/auditor hook (gfx950, wave64):
//   round_planes : FP64 -> FP32 rounding + logging decision, decisions as two dense bit-planes
//   seg_count / seg_scan / compact : ordered stream compaction of the planes into the log
//   replay       : auditor-side re-rounding from the log (primitive "rev")
//   stats        : threshold statistics over two results (Algorithm "threshold", collection)
#include "vt_device.h"
#include "vt_kernels.h"
#include "vt_scan.h"

namespace vt {

namespace {

// --------------------------------------------------------------------------------------------
// round_planes: one wave per segment of 4096 outputs, one output per lane per step, so that a
// wave ballot IS the 64-bit plane word.  Loads are issued eight deep.
// --------------------------------------------------------------------------------------------
constexpr int kUnroll = 8;

__global__ __launch_bounds__(256) void round_planes_kernel(const uint64_t *__restrict__ x, uint64_t n,
                                                           uint32_t thr, uint32_t k, uint32_t *__restrict__ y,
                                                           uint64_t *__restrict__ pl_logged,
                                                           uint64_t *__restrict__ pl_dir,
                                                           uint32_t *__restrict__ seg_cnt, uint32_t segs)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t seg = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (seg >= segs) return;
    const uint64_t base = (uint64_t)seg * kSegElems;
    uint64_t my_lg = 0, my_dr = 0;
    for (uint32_t it = 0; it < kSegWords; it += kUnroll) {
        uint64_t v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t e = base + (uint64_t)(it + u) * 64u + lane;
            v[u] = e < n ? __builtin_nontemporal_load(x + e) : kOneBits;
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint64_t e = base + (uint64_t)(it + u) * 64u + lane;
            const Decision d = decide_k(v[u], k);             // k = 0: rounding amount 32
            if (e < n) __builtin_nontemporal_store(d.ybits, y + e);
            const uint64_t lg = ballot(e < n && d.D < thr);
            const uint64_t dr = ballot(d.dir != 0) & lg;
            if (lane == it + u) { my_lg = lg; my_dr = dr; }
        }
    }
    pl_logged[(uint64_t)seg * kSegWords + lane] = my_lg;
    pl_dir[(uint64_t)seg * kSegWords + lane] = my_dr;
    const uint32_t c = wave_sum(popc64(my_lg));
    if (lane == 0) seg_cnt[seg] = c;
}

__global__ __launch_bounds__(256) void seg_count_kernel(const uint64_t *__restrict__ pl_logged, uint64_t words,
                                                        uint32_t *__restrict__ seg_cnt, uint32_t segs)
{
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t seg = blockIdx.x * 4u + (threadIdx.x >> 6);
    if (seg >= segs) return;
    const uint64_t w = (uint64_t)seg * kSegWords + lane;
    const uint32_t c = wave_sum(w < words ? popc64(pl_logged[w]) : 0u);
    if (lane == 0) seg_cnt[seg] = c;
}

// --------------------------------------------------------------------------------------------
// seg_scan: one block; exclusive prefix of the per-segment counts, total to *count, and the
// direction words that two segments (or the end of the log) share are cleared, because the
// compaction ORs its bits into exactly those words.
// --------------------------------------------------------------------------------------------
constexpr int kScanThreads = 1024;

__global__ __launch_bounds__(kScanThreads) void seg_scan_kernel(const uint32_t *__restrict__ seg_cnt,
                                                                uint32_t *__restrict__ seg_off, uint32_t segs,
                                                                uint32_t *__restrict__ dir, uint64_t cap,
                                                                uint64_t *__restrict__ count)
{
    __shared__ uint64_t wave_total[kScanThreads / 64];
    const uint32_t t = threadIdx.x, lane = t & 63u, wv = t >> 6;
    const uint32_t chunk = (segs + kScanThreads - 1) / kScanThreads;
    const uint64_t lo = (uint64_t)t * chunk;
    const uint64_t hi = lo + chunk < segs ? lo + chunk : segs;
    uint64_t sum = 0;
    for (uint64_t s = lo; s < hi; ++s) sum += seg_cnt[s];
    uint64_t incl = sum;                                    // inclusive scan inside the wave, then over the waves
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint64_t up = (uint64_t)__shfl_up((unsigned long long)incl, o, 64);
        if (lane >= (uint32_t)o) incl += up;
    }
    if (lane == 63) wave_total[wv] = incl;
    __syncthreads();
    uint64_t before = 0, total = 0;
#pragma unroll
    for (uint32_t w = 0; w < kScanThreads / 64; ++w) {
        if (w < wv) before += wave_total[w];
        total += wave_total[w];
    }
    uint64_t run = before + incl - sum;
    const uint64_t cap_words = (cap + 31) >> 5;
    for (uint64_t s = lo; s < hi; ++s) {
        const uint32_t c = seg_cnt[s];
        seg_off[s] = (uint32_t)run;                         // total <= n < 2^32
        if (c) {
            const uint64_t w0 = run >> 5, w1 = (run + c - 1) >> 5;
            if (w0 < cap_words) dir[w0] = 0;
            if (w1 < cap_words) dir[w1] = 0;
        }
        run += c;
    }
    if (t == 0) {
        *count = total;
        if (total > cap && cap > 0) dir[(cap - 1) >> 5] = 0;
    }
}

// --------------------------------------------------------------------------------------------
// compact: one wave per segment (64 plane words, 4096 outputs).  Phase 1: every lane owns one
// plane word; an exclusive scan of the words' population counts gives the rank of its first
// logged output, and the lane writes position (12 bits) and direction (bit 15) of each of its
// set bits to LDS at rank, rank + 1, ...  Ranks of neighbouring lanes lie about as far apart as
// a word has bits set, so the LDS array carries four entries of padding per 64 (ranks 64 l of a
// full plane would otherwise all fall into one bank).  Phase 2 emits the entries 256 at a time,
// aligned to multiples of 256 in log position: four consecutive entries per lane (one 16-byte
// index store where the log is aligned), their direction bits gathered over eight lanes into
// whole 32-bit words; only the words a segment shares with its neighbours are OR-ed.
// --------------------------------------------------------------------------------------------
constexpr uint32_t kEntSlots = kSegElems + 4u * (kSegElems / 64u);

__device__ __forceinline__ uint32_t ent_slot(uint32_t rank) { return rank + 4u * (rank >> 6); }

__global__ __launch_bounds__(256) void compact_kernel(const uint64_t *__restrict__ pl_logged,
                                                      const uint64_t *__restrict__ pl_dir, uint64_t words,
                                                      const uint32_t *__restrict__ seg_cnt,
                                                      const uint32_t *__restrict__ seg_off, uint32_t segs,
                                                      uint32_t wpr, uint32_t ncols,
                                                      uint32_t *__restrict__ idx, uint32_t *__restrict__ dir,
                                                      uint64_t cap)
{
    __shared__ uint16_t ent[4][kEntSlots];
    __shared__ uint32_t wbase[4][kSegWords];
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = threadIdx.x >> 6;
    const uint32_t seg = blockIdx.x * 4u + wv;
    if (seg >= segs) return;
    const uint32_t cnt = seg_cnt[seg];
    if (cnt == 0) return;                                   // wave-uniform
    const uint64_t off = seg_off[seg];
    if (off >= cap) return;
    const uint64_t w = (uint64_t)seg * kSegWords + lane;
    uint64_t m = w < words ? pl_logged[w] : 0;
    const uint64_t dword = w < words ? pl_dir[w] : 0;
    {
        const uint64_t row = w / wpr;
        wbase[wv][lane] = (uint32_t)(row * ncols + (w - row * wpr) * 64u);
    }
    // exclusive scan of the population counts over the wave
    const uint32_t c = popc64(m);
    uint32_t incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, o, 64);
        if (lane >= (uint32_t)o) incl += up;
    }
    uint32_t rank = incl - c;
    while (m) {                                             // lanes leave as their word runs out of bits
        const uint32_t b = (uint32_t)__builtin_ctzll(m);
        ent[wv][ent_slot(rank)] = (uint16_t)((lane << 6) | b | (((uint32_t)(dword >> b) & 1u) << 15));
        m &= m - 1;
        ++rank;
    }
    wave_lds_fence();
    const uint64_t end = off + cnt < cap ? off + cnt : cap;
    const bool wide = ((uintptr_t)idx & 15u) == 0;
    for (uint64_t G = off & ~255ull; G < end; G += 256) {
        const uint64_t p0 = G + 4u * lane;
        uint32_t iv[4], nib_v = 0, nib_d = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t p = p0 + j;
            const bool valid = p >= off && p < end;
            const uint32_t e = valid ? ent[wv][ent_slot((uint32_t)(p - off))] : 0u;
            iv[j] = wbase[wv][(e & 0xFFFu) >> 6] + (e & 63u);
            nib_v |= (uint32_t)valid << j;
            nib_d |= (e >> 15) << j;                        // (e is 0 for invalid positions)
        }
        if (wide && nib_v == 0xFu) {
            *(uint4 *)(idx + p0) = make_uint4(iv[0], iv[1], iv[2], iv[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((nib_v >> j) & 1u) idx[p0 + j] = iv[j];
        }
        // eight lanes' nibbles make one direction word (entries G + 32 g .. G + 32 g + 31)
        uint32_t vv = nib_v << (4u * (lane & 7u)), dv = nib_d << (4u * (lane & 7u));
#pragma unroll
        for (int o = 1; o < 8; o <<= 1) {
            vv |= (uint32_t)__shfl_xor((int)vv, o, 64);
            dv |= (uint32_t)__shfl_xor((int)dv, o, 64);
        }
        if ((lane & 7u) == 0 && vv) {
            uint32_t *wp = dir + (G >> 5) + (lane >> 3);
            if (vv == 0xFFFFFFFFu) *wp = dv;
            else atomicOr(wp, dv);
        }
    }
}

// --------------------------------------------------------------------------------------------
// compact, single launch: the same compaction without the count and scan kernels before it (the
// three launches cost more in the gaps between them than in themselves: about 8 us per kernel
// boundary behind a 0.6 ms GEMM).  A tile is the four segments of a workgroup; it counts its own
// entries, trades the count for its offset with the scanner workgroup (vt_scan.h) while it already
// sorts its entries into LDS, and then emits them as compact_kernel does.  The status words, the
// error words and the direction words of the log must be zero at launch (the producer of the planes
// clears them); the scanner writes *count.
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compact_onepass_kernel(const uint64_t *__restrict__ pl_logged,
                                                              const uint64_t *__restrict__ pl_dir, uint64_t words,
                                                              uint32_t segs, uint32_t wpr, uint32_t ncols,
                                                              uint64_t *__restrict__ st, uint32_t tiles,
                                                              uint32_t *__restrict__ err,
                                                              uint32_t *__restrict__ idx, uint32_t *__restrict__ dir,
                                                              uint64_t cap, uint64_t *__restrict__ count)
{
    __shared__ uint16_t ent[4][kEntSlots];
    __shared__ uint32_t wbase[4][kSegWords];
    __shared__ uint32_t s_cnt[4], s_scan[8];
    __shared__ uint64_t s_off;
    __shared__ uint32_t s_ok;
    if (blockIdx.x == 0) {
        scanner(st, tiles, err, count, s_scan);
        return;
    }
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wv = threadIdx.x >> 6;
    const uint32_t tile = blockIdx.x - 1u;
    const uint32_t seg = tile * 4u + wv;
    const uint64_t w = (uint64_t)seg * kSegWords + lane;
    const bool have = seg < segs && w < words;
    uint64_t m = have ? pl_logged[w] : 0;
    const uint64_t dword = have ? pl_dir[w] : 0;
    {
        const uint64_t row = w / wpr;
        wbase[wv][lane] = (uint32_t)(row * ncols + (w - row * wpr) * 64u);
    }
    // exclusive scan of the population counts over the wave
    const uint32_t c = popc64(m);
    uint32_t incl = c;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t up = (uint32_t)__shfl_up((int)incl, o, 64);
        if (lane >= (uint32_t)o) incl += up;
    }
    const uint32_t cnt = (uint32_t)__shfl((int)incl, 63, 64);      // this segment's entries
    if (lane == 0) s_cnt[wv] = cnt;
    __syncthreads();
    const uint32_t tile_cnt = s_cnt[0] + s_cnt[1] + s_cnt[2] + s_cnt[3];
    if (wv == 0) {
        // publish the tile's count and wait for its place in the log while the other waves sort
        uint64_t off;
        const bool ok = tile_offset(st, tile, tile_cnt, err, lane, off);
        if (lane == 0) { s_off = off; s_ok = ok ? 1u : 0u; }
    }
    uint32_t rank = incl - c;
    while (m) {                                             // lanes leave as their word runs out of bits
        const uint32_t b = (uint32_t)__builtin_ctzll(m);
        ent[wv][ent_slot(rank)] = (uint16_t)((lane << 6) | b | (((uint32_t)(dword >> b) & 1u) << 15));
        m &= m - 1;
        ++rank;
    }
    __syncthreads();
    if (!s_ok || cnt == 0) return;
    uint64_t off = s_off;
#pragma unroll
    for (uint32_t v = 0; v < 3; ++v)
        if (v < wv) off += s_cnt[v];
    if (off >= cap) return;
    const uint64_t end = off + cnt < cap ? off + cnt : cap;
    const bool wide = ((uintptr_t)idx & 15u) == 0;
    for (uint64_t G = off & ~255ull; G < end; G += 256) {
        const uint64_t p0 = G + 4u * lane;
        uint32_t iv[4], nib_v = 0, nib_d = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint64_t p = p0 + j;
            const bool valid = p >= off && p < end;
            const uint32_t e = valid ? ent[wv][ent_slot((uint32_t)(p - off))] : 0u;
            iv[j] = wbase[wv][(e & 0xFFFu) >> 6] + (e & 63u);
            nib_v |= (uint32_t)valid << j;
            nib_d |= (e >> 15) << j;                        // (e is 0 for invalid positions)
        }
        if (wide && nib_v == 0xFu) {
            *(uint4 *)(idx + p0) = make_uint4(iv[0], iv[1], iv[2], iv[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if ((nib_v >> j) & 1u) idx[p0 + j] = iv[j];
        }
        // eight lanes' nibbles make one direction word (entries G + 32 g .. G + 32 g + 31); the words
        // were cleared before the launch, so partial ones are OR-ed
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

// --------------------------------------------------------------------------------------------
// replay: one workgroup per 4096 outputs, each wave a contiguous 1024 (16-byte loads, eight in
// flight).  The first log entry of the tile is found with one 64-ary search of the sorted index
// list; the tile's entries are then read in order and dropped into a byte array in LDS (index
// values are distinct, so plain stores suffice), from which every output picks its own flag.
// --------------------------------------------------------------------------------------------
// A position a with a <= lower_bound(idx, target) <= a + 3, found by one wavefront.  `guess` is
// where the bound would be if the entries were spread evenly; a first round probes 64 positions,
// 256 apart, around it, and when they bracket the bound (the usual case) one more round ends the
// search; otherwise the 64-ary search runs on whatever range remains.  Every read is in bounds.
constexpr uint64_t kProbeGap = 256, kProbeWindow = 64 * kProbeGap;

__device__ __forceinline__ uint64_t wave_lower_bound(const uint32_t *__restrict__ idx, uint64_t count,
                                                     uint64_t target, uint64_t guess, uint32_t lane)
{
    uint64_t a = 0, b = count;                              // answer in [a, b]
    if (count > kProbeWindow) {
        uint64_t a0 = guess > kProbeWindow / 2 ? guess - kProbeWindow / 2 : 0;
        if (a0 + kProbeWindow > count) a0 = count - kProbeWindow;
        const uint32_t c = popc64(ballot((uint64_t)idx[a0 + (uint64_t)lane * kProbeGap] < target));
        if (c == 0) b = a0;
        else {
            a = a0 + (uint64_t)(c - 1) * kProbeGap + 1;
            if (c < 64) b = a0 + (uint64_t)c * kProbeGap;
        }
    }
    while (b - a > 3) {
        const uint64_t step = (b - a + 63) >> 6;
        const uint64_t q = a + (uint64_t)lane * step;
        const bool pred = q < b && (uint64_t)idx[q] < target;
        const uint32_t c = popc64(ballot(pred));
        if (c == 0) { b = a; break; }
        const uint64_t nb = a + (uint64_t)c * step;
        a = a + (uint64_t)(c - 1) * step + 1;
        b = nb < b ? nb : b;
    }
    return a;
}

typedef double d2 __attribute__((ext_vector_type(2)));
typedef float f2 __attribute__((ext_vector_type(2)));

constexpr int kReplayTile = 4096;
constexpr int kReplayChunk = 1024;       // per wave: 8 rows of 128
constexpr int kReplayRows = 8;

template <bool FULL, bool VEC>
__device__ __forceinline__ void replay_load(const double *__restrict__ x, uint64_t n, uint64_t wbase, uint32_t lane,
                                            d2 (&v)[kReplayRows])
{
#pragma unroll
    for (int u = 0; u < kReplayRows; ++u) {
        const uint64_t e = wbase + (uint64_t)u * 128u + 2u * lane;
        if (VEC && (FULL || e + 1 < n)) v[u] = __builtin_nontemporal_load((const d2 *)(x + e));
        else {
            v[u].x = e < n ? x[e] : 1.0;
            v[u].y = e + 1 < n ? x[e + 1] : 1.0;
        }
    }
}

template <bool FULL, bool VEC, bool K0>
__device__ __forceinline__ void replay_store(const d2 (&v)[kReplayRows], const uint8_t *__restrict__ flags,
                                             uint32_t wv, float *__restrict__ y, uint64_t n, uint64_t wbase,
                                             uint32_t lane, uint32_t k)
{
#pragma unroll
    for (int u = 0; u < kReplayRows; ++u) {
        const uint32_t pos = wv * kReplayChunk + (uint32_t)u * 128u + 2u * lane;
        const uint64_t e = wbase + (uint64_t)u * 128u + 2u * lane;
        const uint32_t f = *(const uint16_t *)(flags + pos);          // flags of both outputs
        uint32_t ya, yb;
        if (K0) {
            const FastDecision a = decide_fast(v[u].x), b = decide_fast(v[u].y);
            ya = __float_as_uint(a.y);
            yb = __float_as_uint(b.y);
            if (__builtin_expect(ballot(a.slow || b.slow || f != 0) != 0, 0)) {
                const uint64_t xa = (uint64_t)__double_as_longlong(v[u].x), xb = (uint64_t)__double_as_longlong(v[u].y);
                if (f & 1u) ya = directed(xa, (f >> 1) & 1u);
                else if (a.slow && v[u].x != 0.0) ya = decide(xa).ybits;      // (+-0: the conversion stands)
                if (f & 0x100u) yb = directed(xb, (f >> 9) & 1u);
                else if (b.slow && v[u].y != 0.0) yb = decide(xb).ybits;
            }
        } else {                                                     // rounding amount below 32
            const uint64_t xa = (uint64_t)__double_as_longlong(v[u].x), xb = (uint64_t)__double_as_longlong(v[u].y);
            ya = (f & 1u) ? directed_k(xa, (f >> 1) & 1u, k) : decide_k(xa, k).ybits;
            yb = (f & 0x100u) ? directed_k(xb, (f >> 9) & 1u, k) : decide_k(xb, k).ybits;
        }
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
}

template <bool VEC, bool K0>
__global__ __launch_bounds__(256) void replay_kernel(const double *__restrict__ x, uint64_t n,
                                                     const uint32_t *__restrict__ idx,
                                                     const uint32_t *__restrict__ dir, uint64_t count,
                                                     float *__restrict__ y, uint32_t k)
{
    __shared__ __attribute__((aligned(16))) uint8_t flags[kReplayTile];   // bit 0: logged, bit 1: direction
    __shared__ uint64_t s_lo;
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
    // Consecutive workgroup ids run on different XCDs (8, each with its own L2).  Every XCD takes
    // runs of 64 consecutive tiles, so the index-list lines that the searches of neighbouring tiles
    // share are fetched into one L2 instead of eight, while the eight XCDs together still sweep one
    // window of 512 tiles at a time (an eighth of the array per XCD, eight streams far apart, measured
    // 4 % slower for a plain copy).  The last, incomplete window is walked in id order.
    uint32_t tile = blockIdx.x;
    {
        constexpr uint32_t kRun = 64;
        const uint32_t i = blockIdx.x, window = i / (8u * kRun);
        if ((window + 1u) * (8u * kRun) <= gridDim.x) tile = window * (8u * kRun) + (i % 8u) * kRun + (i / 8u) % kRun;
    }
    const uint64_t start = (uint64_t)tile * kReplayTile;
    const uint64_t stop = start + kReplayTile < n ? start + kReplayTile : n;
    const uint64_t wbase = start + (uint64_t)wv * kReplayChunk;
    const bool full = start + kReplayTile <= n;
    d2 v[kReplayRows];
    if (full) replay_load<true, VEC>(x, n, wbase, lane, v);
    else replay_load<false, VEC>(x, n, wbase, lane, v);
    ((uint4 *)flags)[tid] = make_uint4(0, 0, 0, 0);
    if (wv == 0) {
        const double even = (double)start * ((double)count / (double)n);
        const uint64_t r = wave_lower_bound(idx, count, start, even < (double)count ? (uint64_t)even : count, lane);
        if (lane == 0) s_lo = r;
    }
    __syncthreads();
    const uint64_t lo = s_lo;
    // lo is at most 3 before the tile's first entry, and at most 4096 entries belong to the tile:
    // 64 rounds of 64 plus one for the ragged start
    // (a wave takes rounds wv, wv + 4, ...; four of its rounds are requested together, so that a tile
    // with many entries pays one memory round trip per 16 rounds instead of one per 4)
    for (uint32_t r0 = wv; r0 <= kReplayTile / 64; r0 += 16) {
        uint64_t pp[4], ii[4];
        uint32_t dd[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const uint32_t r = r0 + 4u * (uint32_t)q;
            pp[q] = lo + (uint64_t)r * 64u + lane;
            const bool in = r <= kReplayTile / 64 && pp[q] < count;
            ii[q] = in ? (uint64_t)idx[pp[q]] : ~0ull;
            dd[q] = in ? dir[pp[q] >> 5] : 0u;
        }
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (ii[q] >= start && ii[q] < stop)
                flags[ii[q] - start] = (uint8_t)(1u | (((dd[q] >> (pp[q] & 31u)) & 1u) << 1));
        if (ballot(ii[3] < stop) == 0) break;                // sorted list: nothing further belongs here
    }
    __syncthreads();
    if (full) replay_store<true, VEC, K0>(v, flags, wv, y, n, wbase, lane, k);
    else replay_store<false, VEC, K0>(v, flags, wv, y, n, wbase, lane, k);
}

// --------------------------------------------------------------------------------------------
// stats: grid-stride, integer reductions only (sums and maxima commute exactly, so the result
// does not depend on scheduling).
// --------------------------------------------------------------------------------------------
__global__ void fill_u64_kernel(uint64_t *p, uint32_t nwords, uint64_t v)
{
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = v;
}

// Persistent grid (few workgroups, so few global atomics at the end), 16-byte loads, eight in
// flight per lane.  The histogram lives in LDS in 16 copies selected by lane, which keeps
// same-address collisions of the LDS atomics short; identical pairs (bin 0) are only counted.
constexpr int kStatsU = 4;                      // 16-byte loads per array, lane and iteration
constexpr int kStatsTile = 256 * 2 * kStatsU;   // elements per workgroup and iteration

struct StatsAcc {
    uint32_t flips, thrmax, equal;
    uint64_t dmax;
};

template <bool K0>
__device__ __forceinline__ void stats_one(uint64_t a, uint64_t b, double xa, double xb, bool valid, uint32_t copy,
                                          uint32_t (*hist)[66], StatsAcc &acc, uint32_t k)
{
    if (!valid) return;
    if (a == b) { ++acc.equal; return; }
    const int64_t oa = ord64(a), ob = ord64(b);
    const uint64_t diff = oa > ob ? (uint64_t)oa - (uint64_t)ob : (uint64_t)ob - (uint64_t)oa;
    if (diff == 0) ++acc.equal;                                   // +0 / -0
    else {
        atomicAdd(&hist[copy][64u - (uint32_t)__clzll((long long)diff)], 1u);
        acc.dmax = diff > acc.dmax ? diff : acc.dmax;
    }
    // FP32 roundings: hardware conversion when both values are ordinary (the conversion cannot
    // differ from the integer definition there); distances only for the rare pairs that flip
    const uint32_t ha = (uint32_t)(a >> 32) & 0x7FFFFFFFu, hb = (uint32_t)(b >> 32) & 0x7FFFFFFFu;
    const bool ordinary = (ha - (897u << 20)) < ((1151u - 897u) << 20) && (hb - (897u << 20)) < ((1151u - 897u) << 20);
    if (K0 && ordinary) {
        if (__float_as_uint((float)xa) == __float_as_uint((float)xb)) return;
        const uint32_t Da = __usad((uint32_t)a & kMask29, kHalf, 0u), Db = __usad((uint32_t)b & kMask29, kHalf, 0u);
        ++acc.flips;
        const uint32_t need = 1u + (Da > Db ? Da : Db);
        acc.thrmax = need > acc.thrmax ? need : acc.thrmax;
        return;
    }
    if (!K0 && ordinary && ((a ^ b) >> 63) == 0) {
        // Coarser grids: in the FP32-normal range the grid points are the patterns whose low 29 + k bits
        // are zero, and rounding to nearest is rounding of the pattern; two values of one sign whose
        // patterns round to the same point, neither of them a tie, cannot flip.  (Everything else,
        // the rare pairs, goes through the full decision below.)
        const uint32_t s = 29u + k;
        const uint64_t half = 1ull << (s - 1u), low = (1ull << s) - 1ull;
        const uint64_t ua = (a & 0x7FFFFFFFFFFFFFFFull) + half, ub = (b & 0x7FFFFFFFFFFFFFFFull) + half;
        if ((ua >> s) == (ub >> s) && (ua & low) != 0 && (ub & low) != 0) return;
    }
    const Decision da = decide_k(a, k), db = decide_k(b, k);
    if (da.ybits != db.ybits) {
        ++acc.flips;
        const uint32_t need = 1u + (da.D > db.D ? da.D : db.D);
        acc.thrmax = need > acc.thrmax ? need : acc.thrmax;
    }
}

template <bool VEC, bool K0>
__global__ __launch_bounds__(256) void stats_kernel(const double *__restrict__ y1, const double *__restrict__ y2,
                                                    uint64_t n, uint64_t *__restrict__ out, uint32_t k)
{
    __shared__ uint32_t hist[16][66];
    __shared__ unsigned long long s_flip, s_thr, s_max, s_eq;
    const uint32_t tid = threadIdx.x, copy = tid & 15u;
    for (uint32_t k = tid; k < 16 * 66; k += 256) (&hist[0][0])[k] = 0;
    if (tid == 0) { s_flip = 0; s_thr = 0; s_max = 0; s_eq = 0; }
    __syncthreads();
    StatsAcc acc = {0, 0, 0, 0};
    for (uint64_t base = (uint64_t)blockIdx.x * kStatsTile; base < n; base += (uint64_t)gridDim.x * kStatsTile) {
        d2 a[kStatsU], b[kStatsU];
        const bool full = base + kStatsTile <= n;
#pragma unroll
        for (int u = 0; u < kStatsU; ++u) {
            const uint64_t e = base + (uint64_t)u * 512u + 2u * tid;
            if (VEC && (full || e + 1 < n)) {
                a[u] = __builtin_nontemporal_load((const d2 *)(y1 + e));
                b[u] = __builtin_nontemporal_load((const d2 *)(y2 + e));
            } else {
                a[u].x = e < n ? y1[e] : 0.0;      a[u].y = e + 1 < n ? y1[e + 1] : 0.0;
                b[u].x = e < n ? y2[e] : 0.0;      b[u].y = e + 1 < n ? y2[e + 1] : 0.0;
            }
        }
#pragma unroll
        for (int u = 0; u < kStatsU; ++u) {
            const uint64_t e = base + (uint64_t)u * 512u + 2u * tid;
            stats_one<K0>((uint64_t)__double_as_longlong(a[u].x), (uint64_t)__double_as_longlong(b[u].x), a[u].x, b[u].x,
                          full || e < n, copy, hist, acc, k);
            stats_one<K0>((uint64_t)__double_as_longlong(a[u].y), (uint64_t)__double_as_longlong(b[u].y), a[u].y, b[u].y,
                          full || e + 1 < n, copy, hist, acc, k);
        }
    }
    atomicAdd(&s_flip, (unsigned long long)acc.flips);
    atomicAdd(&s_eq, (unsigned long long)acc.equal);
    atomicMax(&s_thr, (unsigned long long)acc.thrmax);
    atomicMax(&s_max, (unsigned long long)acc.dmax);
    __syncthreads();
    if (tid < 65) {
        unsigned long long h = tid == 0 ? s_eq : 0ull;
#pragma unroll
        for (int c = 0; c < 16; ++c) h += hist[c][tid];
        if (h) atomicAdd((unsigned long long *)&out[3 + tid], h);
    }
    if (tid == 0) {
        if (s_flip) atomicAdd((unsigned long long *)&out[0], s_flip);
        if (s_thr) atomicMax((unsigned long long *)&out[1], s_thr);
        if (s_max) atomicMax((unsigned long long *)&out[2], s_max);
    }
}

}  // namespace

// ------------------------------------------------------------------------------------ host side

static uint64_t round_up(uint64_t v, uint64_t a) { return (v + a - 1) / a * a; }

size_t planes_bytes(uint64_t rows, uint64_t ncols)
{
    const uint64_t wpr = (ncols + 63) / 64;
    const uint64_t words = rows * wpr;
    const uint64_t segs = (words + kSegWords - 1) / kSegWords;
    return (size_t)(2 * round_up(segs * kSegWords * 8, 256) + 2 * round_up(segs * 4, 256));
}

Planes planes_carve(void *ws, uint64_t rows, uint64_t ncols)
{
    Planes p;
    const uint64_t wpr = (ncols + 63) / 64;
    p.words = rows * wpr;
    p.segs = (uint32_t)((p.words + kSegWords - 1) / kSegWords);
    p.wpr = (uint32_t)(wpr ? wpr : 1);
    p.ncols = (uint32_t)ncols;
    char *c = (char *)ws;
    const uint64_t plane = round_up((uint64_t)p.segs * kSegWords * 8, 256);
    const uint64_t segarr = round_up((uint64_t)p.segs * 4, 256);
    p.logged = (uint64_t *)c;
    p.dir = (uint64_t *)(c + plane);
    p.seg_cnt = (uint32_t *)(c + 2 * plane);
    p.seg_off = (uint32_t *)(c + 2 * plane + segarr);
    return p;
}

hipError_t launch_round_planes(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, const Planes &pl,
                               hipStream_t s)
{
    if (pl.segs == 0) return hipSuccess;
    round_planes_kernel<<<(pl.segs + 3) / 4, 256, 0, s>>>((const uint64_t *)x, n, thr, k, (uint32_t *)y, pl.logged,
                                                         pl.dir, pl.seg_cnt, pl.segs);
    return hipGetLastError();
}

hipError_t launch_seg_count(const Planes &pl, hipStream_t s)
{
    if (pl.segs == 0) return hipSuccess;
    seg_count_kernel<<<(pl.segs + 3) / 4, 256, 0, s>>>(pl.logged, pl.words, pl.seg_cnt, pl.segs);
    return hipGetLastError();
}

hipError_t launch_seg_scan(const Planes &pl, const LogOut &log, hipStream_t s)
{
    seg_scan_kernel<<<1, kScanThreads, 0, s>>>(pl.seg_cnt, pl.seg_off, pl.segs, log.dir, log.cap, log.count);
    return hipGetLastError();
}

void compact_onepass_scratch(const Planes &pl, uint32_t **zero, uint32_t *zero_words)
{
    const uint32_t tiles = (pl.segs + 3u) / 4u;
    *zero = pl.seg_cnt;                                     // status words (8 bytes per tile), then the error words
    *zero_words = 2u * tiles + 4u;
}

hipError_t launch_compact_onepass(const Planes &pl, const LogOut &log, hipStream_t s)
{
    if (pl.segs == 0) return hipErrorInvalidValue;
    const uint32_t tiles = (pl.segs + 3u) / 4u;
    uint64_t *st = (uint64_t *)pl.seg_cnt;
    uint32_t *err = (uint32_t *)(st + tiles);
    compact_onepass_kernel<<<tiles + 1u, 256, 0, s>>>(pl.logged, pl.dir, pl.words, pl.segs, pl.wpr, pl.ncols, st, tiles, err,
                                                      log.idx, log.dir, log.cap, log.count);
    return hipGetLastError();
}

hipError_t launch_compact(const Planes &pl, const LogOut &log, hipStream_t s)
{
    if (pl.segs == 0 || log.cap == 0) return hipSuccess;
    compact_kernel<<<(pl.segs + 3) / 4, 256, 0, s>>>(pl.logged, pl.dir, pl.words, pl.seg_cnt, pl.seg_off, pl.segs,
                                                    pl.wpr, pl.ncols, log.idx, log.dir, log.cap);
    return hipGetLastError();
}

hipError_t launch_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir, uint64_t count,
                         uint32_t k, float *y, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kReplayTile - 1) / kReplayTile;
    const bool vec = ((uintptr_t)x % 16 == 0) && ((uintptr_t)y % 8 == 0);
    const dim3 grid((uint32_t)blocks), block(256);
    if (vec && k == 0) replay_kernel<true, true><<<grid, block, 0, s>>>(x, n, idx, dir, count, y, k);
    else if (vec) replay_kernel<true, false><<<grid, block, 0, s>>>(x, n, idx, dir, count, y, k);
    else if (k == 0) replay_kernel<false, true><<<grid, block, 0, s>>>(x, n, idx, dir, count, y, k);
    else replay_kernel<false, false><<<grid, block, 0, s>>>(x, n, idx, dir, count, y, k);
    return hipGetLastError();
}

hipError_t launch_stats(const double *y1, const double *y2, uint64_t n, uint32_t k, uint64_t *out, hipStream_t s)
{
    fill_u64_kernel<<<1, 128, 0, s>>>(out, 68, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    uint64_t blocks = (n + kStatsTile - 1) / kStatsTile;
    // 4 workgroups per CU keep enough loads in flight for the HBM rate; 8 per CU double the burst
    // of final atomics (measured slower at every size).
    if (blocks > 1024) blocks = 1024;
    const bool vec = ((uintptr_t)y1 % 16 == 0) && ((uintptr_t)y2 % 16 == 0);
    const dim3 grid((uint32_t)blocks), block(256);
    if (vec && k == 0) stats_kernel<true, true><<<grid, block, 0, s>>>(y1, y2, n, out, k);
    else if (vec) stats_kernel<true, false><<<grid, block, 0, s>>>(y1, y2, n, out, k);
    else if (k == 0) stats_kernel<false, true><<<grid, block, 0, s>>>(y1, y2, n, out, k);
    else stats_kernel<false, false><<<grid, block, 0, s>>>(y1, y2, n, out, k);
    return hipGetLastError();
}

}  // namespace vt
