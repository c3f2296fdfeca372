// vt_round_kernels.hip -- HBM-bound kernels of the trainer/auditor hook (gfx950, wave64):
//   round_planes : FP64 -> FP32 rounding + logging decision, decisions as two dense bit-planes
//   seg_count / seg_scan / compact : ordered stream compaction of the planes into the log
//   replay       : auditor-side re-rounding from the log (primitive "rev")
//   stats        : threshold statistics over two results (Algorithm "threshold", collection)
#include "vt_device.h"
#include "vt_kernels.h"

namespace vt {

namespace {

// --------------------------------------------------------------------------------------------
// round_planes: one wave per segment of 4096 outputs, one output per lane per step, so that a
// wave ballot IS the 64-bit plane word.  Loads are issued eight deep.
// --------------------------------------------------------------------------------------------
constexpr int kUnroll = 8;

__global__ __launch_bounds__(256) void round_planes_kernel(const uint64_t *__restrict__ x, uint64_t n,
                                                           uint32_t thr, uint32_t *__restrict__ y,
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
            const Decision d = decide(v[u]);
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
    __shared__ uint64_t part[kScanThreads];
    const uint32_t t = threadIdx.x;
    const uint32_t chunk = (segs + kScanThreads - 1) / kScanThreads;
    const uint64_t lo = (uint64_t)t * chunk;
    const uint64_t hi = lo + chunk < segs ? lo + chunk : segs;
    uint64_t sum = 0;
    for (uint64_t s = lo; s < hi; ++s) sum += seg_cnt[s];
    part[t] = sum;
    __syncthreads();
    for (int o = 1; o < kScanThreads; o <<= 1) {           // inclusive Hillis-Steele scan
        const uint64_t add = t >= (uint32_t)o ? part[t - o] : 0;
        __syncthreads();
        part[t] += add;
        __syncthreads();
    }
    const uint64_t total = part[kScanThreads - 1];
    uint64_t run = part[t] - sum;
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
// compact: one wave per segment.  Phase 1 walks the 64 plane words (skipping empty ones) and
// writes each logged output's position inside the segment (12 bits) and direction (bit 15) to
// LDS at its rank.  Phase 2 emits entries 64 at a time, aligned to multiples of 64 in log
// position, so index stores are contiguous and a ballot yields whole direction words.
// --------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void compact_kernel(const uint64_t *__restrict__ pl_logged,
                                                      const uint64_t *__restrict__ pl_dir, uint64_t words,
                                                      const uint32_t *__restrict__ seg_cnt,
                                                      const uint32_t *__restrict__ seg_off, uint32_t segs,
                                                      uint32_t wpr, uint32_t ncols,
                                                      uint32_t *__restrict__ idx, uint32_t *__restrict__ dir,
                                                      uint64_t cap)
{
    __shared__ uint16_t ent[4][kSegElems];
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
    const uint64_t word = w < words ? pl_logged[w] : 0;
    const uint64_t dword = w < words ? pl_dir[w] : 0;
    {
        const uint64_t row = w / wpr;
        wbase[wv][lane] = (uint32_t)(row * ncols + (w - row * wpr) * 64u);
    }
    uint32_t local = 0;
    for (uint32_t i = 0; i < kSegWords; ++i) {
        const uint64_t m = readlane64(word, i);
        if (m == 0) continue;
        const uint64_t d = readlane64(dword, i);
        if ((m >> lane) & 1ull)
            ent[wv][local + rank_below(m)] = (uint16_t)((i << 6) | lane | (((uint32_t)(d >> lane) & 1u) << 15));
        local += popc64(m);
    }
    wave_lds_fence();
    const uint64_t end = off + cnt < cap ? off + cnt : cap;
    for (uint64_t G = off & ~63ull; G < end; G += 64) {
        const uint64_t p = G + lane;
        const bool valid = p >= off && p < end;
        const uint32_t e = valid ? ent[wv][p - off] : 0u;
        if (valid) idx[p] = wbase[wv][(e & 0xFFFu) >> 6] + (e & 63u);
        const uint64_t dm = ballot(valid && (e >> 15));
        const uint64_t vm = ballot(valid);
        if (lane < 2) {
            const uint32_t vh = lane ? (uint32_t)(vm >> 32) : (uint32_t)vm;
            const uint32_t dh = lane ? (uint32_t)(dm >> 32) : (uint32_t)dm;
            uint32_t *wp = dir + (G >> 5) + lane;
            if (vh == 0xFFFFFFFFu) *wp = dh;
            else if (vh) atomicOr(wp, dh);
        }
    }
}

// --------------------------------------------------------------------------------------------
// replay: one block per 4096 outputs.  The block's slice of the sorted log is found with two
// 64-ary searches (one wave each), scattered into LDS bit arrays, then the outputs are streamed.
// --------------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t wave_lower_bound(const uint32_t *__restrict__ idx, uint64_t count,
                                                     uint64_t target, uint32_t lane)
{
    uint64_t a = 0, b = count;                              // answer in [a, b]
    while (b > a) {
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

constexpr int kReplayTile = 4096;
constexpr int kReplayPer = kReplayTile / 256;

__global__ __launch_bounds__(256) void replay_kernel(const uint64_t *__restrict__ x, uint64_t n,
                                                     const uint32_t *__restrict__ idx,
                                                     const uint32_t *__restrict__ dir, uint64_t count,
                                                     uint32_t *__restrict__ y)
{
    __shared__ uint32_t s_lg[kReplayTile / 32], s_dr[kReplayTile / 32];
    __shared__ uint64_t s_range[2];
    const uint32_t tid = threadIdx.x, lane = tid & 63u, wv = tid >> 6;
    const uint64_t start = (uint64_t)blockIdx.x * kReplayTile;
    const uint64_t stop = start + kReplayTile < n ? start + kReplayTile : n;
    uint64_t v[kReplayPer];
#pragma unroll
    for (int u = 0; u < kReplayPer; ++u) {
        const uint64_t e = start + (uint64_t)u * 256u + tid;
        v[u] = e < stop ? __builtin_nontemporal_load(x + e) : kOneBits;
    }
    if (tid < kReplayTile / 32) { s_lg[tid] = 0; s_dr[tid] = 0; }
    if (wv < 2) {
        const uint64_t r = wave_lower_bound(idx, count, wv ? stop : start, lane);
        if (lane == 0) s_range[wv] = r;
    }
    __syncthreads();
    const uint64_t lo = s_range[0], hi = s_range[1];
    for (uint64_t p = lo + tid; p < hi; p += 256) {
        const uint64_t i = idx[p];
        if (i >= start && i < stop) {
            const uint32_t o = (uint32_t)(i - start);
            atomicOr(&s_lg[o >> 5], 1u << (o & 31u));
            if ((dir[p >> 5] >> (p & 31u)) & 1u) atomicOr(&s_dr[o >> 5], 1u << (o & 31u));
        }
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kReplayPer; ++u) {
        const uint32_t o = (uint32_t)u * 256u + tid;
        const uint64_t e = start + o;
        const uint32_t lg = (s_lg[o >> 5] >> (o & 31u)) & 1u;
        const uint32_t dr = (s_dr[o >> 5] >> (o & 31u)) & 1u;
        const uint32_t yb = lg ? directed(v[u], dr) : decide(v[u]).ybits;
        if (e < stop) __builtin_nontemporal_store(yb, y + e);
    }
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

__global__ __launch_bounds__(256) void stats_kernel(const uint64_t *__restrict__ y1, const uint64_t *__restrict__ y2,
                                                    uint64_t n, uint64_t *__restrict__ out)
{
    __shared__ uint32_t s_hist[65];
    __shared__ unsigned long long s_flip, s_thr, s_max;
    const uint32_t tid = threadIdx.x, lane = tid & 63u;
    if (tid < 65) s_hist[tid] = 0;
    if (tid == 0) { s_flip = 0; s_thr = 0; s_max = 0; }
    __syncthreads();
    uint32_t flips = 0, thrmax = 0;
    uint64_t dmax = 0;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    const uint64_t rounds = (n + stride - 1) / stride;      // uniform trip count: ballots need whole waves
    for (uint64_t rd = 0; rd < rounds; ++rd) {
        const uint64_t i = rd * stride + (uint64_t)blockIdx.x * 256u + tid;
        const bool in = i < n;
        const uint64_t a = in ? __builtin_nontemporal_load(y1 + i) : 0;
        const uint64_t b = in ? __builtin_nontemporal_load(y2 + i) : 0;
        const int64_t oa = ord64(a), ob = ord64(b);
        const uint64_t diff = oa > ob ? (uint64_t)oa - (uint64_t)ob : (uint64_t)ob - (uint64_t)oa;
        uint32_t bin = diff ? 64u - (uint32_t)__clzll((long long)diff) : 0u;
        if (in) {
            dmax = diff > dmax ? diff : dmax;
            if (a != b) {                                   // identical patterns cannot flip (+0 / -0 can)
                const Decision da = decide(a), db = decide(b);
                if (da.ybits != db.ybits) {
                    ++flips;
                    const uint32_t need = 1u + (da.D > db.D ? da.D : db.D);
                    thrmax = need > thrmax ? need : thrmax;
                }
            }
        }
        // histogram: one LDS atomic per distinct bin per wave
        uint64_t todo = ballot(in);
        while (todo) {
            const uint32_t leader = (uint32_t)__builtin_ctzll(todo);
            const uint32_t lb = (uint32_t)__builtin_amdgcn_readlane((int)bin, (int)leader);
            const uint64_t same = ballot(in && bin == lb) & todo;
            if (lane == leader) atomicAdd(&s_hist[lb], popc64(same));
            todo &= ~same;
        }
    }
    atomicAdd(&s_flip, (unsigned long long)flips);
    atomicMax(&s_thr, (unsigned long long)thrmax);
    atomicMax(&s_max, (unsigned long long)dmax);
    __syncthreads();
    if (tid < 65 && s_hist[tid]) atomicAdd((unsigned long long *)&out[3 + tid], (unsigned long long)s_hist[tid]);
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

hipError_t launch_round_planes(const double *x, uint64_t n, uint32_t thr, float *y, const Planes &pl, hipStream_t s)
{
    if (pl.segs == 0) return hipSuccess;
    round_planes_kernel<<<(pl.segs + 3) / 4, 256, 0, s>>>((const uint64_t *)x, n, thr, (uint32_t *)y, pl.logged,
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

hipError_t launch_compact(const Planes &pl, const LogOut &log, hipStream_t s)
{
    if (pl.segs == 0 || log.cap == 0) return hipSuccess;
    compact_kernel<<<(pl.segs + 3) / 4, 256, 0, s>>>(pl.logged, pl.dir, pl.words, pl.seg_cnt, pl.seg_off, pl.segs,
                                                    pl.wpr, pl.ncols, log.idx, log.dir, log.cap);
    return hipGetLastError();
}

hipError_t launch_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir, uint64_t count,
                         float *y, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    const uint64_t blocks = (n + kReplayTile - 1) / kReplayTile;
    replay_kernel<<<(uint32_t)blocks, 256, 0, s>>>((const uint64_t *)x, n, idx, dir, count, (uint32_t *)y);
    return hipGetLastError();
}

hipError_t launch_stats(const double *y1, const double *y2, uint64_t n, uint64_t *out, hipStream_t s)
{
    fill_u64_kernel<<<1, 128, 0, s>>>(out, 68, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || n == 0) return e;
    uint64_t blocks = (n + 256 * 8 - 1) / (256 * 8);
    if (blocks > 16384) blocks = 16384;
    stats_kernel<<<(uint32_t)blocks, 256, 0, s>>>((const uint64_t *)y1, (const uint64_t *)y2, n, out);
    return hipGetLastError();
}

}  // namespace vt
