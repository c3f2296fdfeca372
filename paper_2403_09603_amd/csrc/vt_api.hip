// vt_api.hip -- the C ABI declared in include/vt.h: argument checks and kernel sequencing.
#include "../../include/vt.h"
#include "vt_conv_phases.h"
#include "vt_kernels.h"

#include <atomic>
#include <cmath>

// Scratch of vt_round_log_static: the status words of the one-pass kernel (8 bytes per tile of 4096
// outputs, then its error words) or the 256 spread counters of the packed-log kernel.  One copy per
// GPU, held until the process ends; in host code the name is only a handle for hipGetSymbolAddress.
#define VT_STATIC_SCRATCH_BYTES ((VT_ROUND_LOG_STATIC_MAX_N / 4096) * 8 + 16384)
static __device__ __align__(256) unsigned char scratch[VT_STATIC_SCRATCH_BYTES];

namespace {

// device address of `scratch` on each GPU (every GPU holds its own copy at its own address),
// resolved on the first call made with that GPU current
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];

int static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return VT_ERR_HIP;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return VT_ERR_HIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // (a racing first call resolves the same address)
    }
    *out = p;
    return VT_OK;
}

// Optional instrumentation (vt_set_kernel_events): events recorded around the main kernel.
hipEvent_t g_ev_begin = nullptr, g_ev_end = nullptr;
inline void mark_begin(hipStream_t s) { if (g_ev_begin) (void)hipEventRecord(g_ev_begin, s); }
inline void mark_end(hipStream_t s) { if (g_ev_end) (void)hipEventRecord(g_ev_end, s); }

inline bool aligned(const void *p, size_t a) { return ((uintptr_t)p % a) == 0; }

inline int hip_status(hipError_t e) { return e == hipSuccess ? VT_OK : VT_ERR_HIP; }

inline bool log_ok(const vt_log *log)
{
    if (!log || !log->count || !aligned(log->count, 8)) return false;
    if (log->cap && (!log->idx || !log->dir || !aligned(log->idx, 4) || !aligned(log->dir, 4))) return false;
    if (log->dense && (log->cap || !aligned(log->dense, 4))) return false;      // one format per call
    if (log->b_r != 0 && (log->b_r < 10 || log->b_r > 32)) return false;
    return true;
}

inline bool br_ok(int b_r) { return b_r >= 10 && b_r <= 32; }
inline uint32_t k_of(int b_r) { return b_r == 0 ? 0u : (uint32_t)(32 - b_r); }   // zeroed low mantissa bits

inline size_t round_log_bytes(uint64_t n)
{
    const size_t a = vt::planes_bytes(1, n), b = vt::onepass_bytes(n), c = vt::dense_count_bytes();
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

// the larger split factor of the two operand layouts (the workspace query does not know which)
inline int max_splits(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    int most = 1;
    for (int layout : {vt::kALayoutRowMajor, vt::kALayoutTransposed, vt::kALayoutIm2colT}) {
        const int sp = vt::plan_gemm(M, N, K < 0 ? 0 : K, batch, true, layout).splits;
        most = sp > most ? sp : most;
    }
    return most;
}

// scratch for the slices of tail tiles (gemm_tail_cut) under any plan this shape can get: the workspace query
// knows neither the operand layout nor whether the output is dense
inline size_t tail_bytes_for(int64_t M, int64_t N, int64_t K, int64_t batch)
{
    size_t most = 0;
    if (M <= 0 || N <= 0 || K <= 0 || batch <= 0) return 0;
    for (int layout : {vt::kALayoutRowMajor, vt::kALayoutTransposed, vt::kALayoutIm2colT})
        for (bool allow : {false, true}) {
            const vt::GemmPlan plan = vt::plan_gemm(M, N, K, batch, allow, layout);
            if (plan.splits != 1) continue;
            const int64_t t = plan.shape == 0 ? 128 : 64;
            const uint64_t tiles = (uint64_t)((M + t - 1) / t) * (uint64_t)((N + t - 1) / t) * (uint64_t)batch;
            if (!vt::gemm_tail_cut(plan.shape, tiles, (K + 15) / 16)) continue;
            const size_t bytes = (size_t)(tiles % 256u) * 4u * (size_t)(t * t * 8);
            most = bytes > most ? bytes : most;
        }
    return most;
}

inline bool split_allowed(int64_t M, int64_t N, int64_t batch, int64_t ldc, int64_t strideC)
{
    return ldc == N && (batch <= 1 || strideC == M * N);    // the round/log pass sees one flat tensor
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }

// Input gradient of a convolution: offset of the re-laid filter in the workspace.  Below it lies
// either the GEMM's own workspace (one GEMM over the whole view) or, for a strided layer computed
// phase by phase, the round/log scratch and the phases' FP64 results.
inline size_t dgrad_filter_offset(int64_t M, int64_t N, int64_t K, bool two_pass)
{
    const size_t gemm = vt_workspace_bytes(two_pass ? VT_OP_GEMM_ROUND_LOG_BR : VT_OP_GEMM_ROUND_LOG, M, N, K, 1);
    const uint64_t total = (uint64_t)M * (uint64_t)N;
    const size_t phased = up256(round_log_bytes(total)) + up256((size_t)total * 8);
    return up256(gemm > phased ? gemm : phased);
}

// round + log of a flat FP64 tensor that already lives in device memory (trainer hook)
int round_log_flat(const double *x, uint64_t n, uint32_t thr, float *y, const vt_log *log, void *ws, hipStream_t s,
                   bool mark)
{
    const uint32_t k = k_of(log->b_r);
    if (log->dense) {                       // packed ternary log: positional, a plain stream
        if (mark) mark_begin(s);
        const hipError_t e0 = vt::launch_round_log_dense(x, n, thr, k, y, log->dense, log->count, (uint64_t *)ws, s);
        if (mark) mark_end(s);
        return hip_status(e0);
    }
    const vt::LogOut lo{log->idx, log->dir, log->cap, log->count};
    if (thr == 0 && n > 0 && vt::onepass_usable(x, y)) {      // nothing can be logged: round only, count 0
        if (mark) mark_begin(s);
        const hipError_t e0 = vt::launch_round_only(x, n, k, y, log->count, s);
        if (mark) mark_end(s);
        return hip_status(e0);
    }
    if (vt::onepass_usable(x, y)) {         // one streaming pass; otherwise bit-planes + compaction
        if (mark) mark_begin(s);
        const hipError_t e1 = vt::launch_round_log_onepass(x, n, thr, k, y, ws, lo, s);
        if (mark) mark_end(s);
        return hip_status(e1);
    }
    const vt::Planes pl = vt::planes_carve(ws, 1, n);
    if (mark) mark_begin(s);
    hipError_t e = vt::launch_round_planes(x, n, thr, k, y, pl, s);
    if (mark) mark_end(s);
    if (e == hipSuccess) e = vt::launch_seg_scan(pl, lo, s);
    if (e == hipSuccess) e = vt::launch_compact(pl, lo, s);
    return hip_status(e);
}

// planes already hold the decisions: compaction to the ordered log.  `cleared`: the kernel that wrote the
// planes also zeroed what the single-launch compaction needs (see prepare_compaction)
int finish_log(const vt::Planes &pl, uint64_t rows, const vt_log *log, bool cleared, uint32_t thr, hipStream_t s)
{
    if (log->dense) return hip_status(vt::launch_planes_to_dense(pl, rows, log->dense, log->count, s));   // also writes *count
    const vt::LogOut lo{log->idx, log->dir, log->cap, log->count};
    if (thr == 0) {                         // a zero threshold logs nothing (the auditor's own layer): the count is 0
        vt::Planes none = pl;
        none.segs = 0;
        return hip_status(vt::launch_seg_scan(none, lo, s));
    }
    if (cleared) return hip_status(vt::launch_compact_onepass(pl, lo, s));   // also writes *count
    hipError_t e = vt::launch_seg_count(pl, s);
    if (e == hipSuccess) e = vt::launch_seg_scan(pl, lo, s);                 // also writes *count
    if (e == hipSuccess) e = vt::launch_compact(pl, lo, s);
    return hip_status(e);
}

// Tells the GEMM kernel what to zero for the single-launch compaction of an index-list log: the scanner's
// scratch and the direction words the entries will be OR-ed into.  False when that route is not taken.
bool prepare_compaction(vt::GemmArgs &g, const vt::Planes &pl, const vt_log *log, uint64_t total)
{
    if (log->dense || g.thr == 0 || pl.segs == 0) return false;
    vt::compact_onepass_scratch(pl, &g.zero_b, &g.zero_b_words);
    const uint64_t stored = log->cap < total ? log->cap : total;
    g.zero_a = log->dir;
    g.zero_a_words = (uint32_t)((stored + 31) / 32);
    return true;
}

// workspace check, plan, launch and log compaction shared by the GEMM and convolution entry points
int run_gemm(vt::GemmArgs &g, const vt_log *log, void *ws, size_t ws_bytes, hipStream_t s)
{
    const int64_t M = g.M, N = g.N, K = g.K, batch = g.batch;
    const uint64_t total = (uint64_t)M * (uint64_t)N * (uint64_t)batch;
    // a rounding amount below 32 is applied by the standalone hook to the FP64 result in memory
    const bool two_pass = k_of(log->b_r) != 0;
    if (two_pass && !split_allowed(M, N, batch, g.ldc, g.strideC)) return VT_ERR_UNSUPPORTED;
    const size_t need = vt_workspace_bytes(two_pass ? VT_OP_GEMM_ROUND_LOG_BR : VT_OP_GEMM_ROUND_LOG, M, N, K, batch);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return VT_ERR_WORKSPACE;
    const vt::Planes pl = vt::planes_carve(ws, (uint64_t)M * (uint64_t)batch, (uint64_t)N);
    const size_t planes = vt::planes_bytes((uint64_t)M * (uint64_t)batch, (uint64_t)N);
    const int a_layout = g.conv && g.conv_wgrad ? vt::kALayoutIm2colT : (g.transA ? vt::kALayoutTransposed : vt::kALayoutRowMajor);
    const vt::GemmPlan plan = vt::plan_gemm(M, N, K, batch, split_allowed(M, N, batch, g.ldc, g.strideC), a_layout);
    g.raw = two_pass;
    if (plan.splits > 1 || two_pass) {
        // slabs -> fixed-order sum (alpha, bias) -> standalone round/log over the flat result
        double *partial = (double *)((char *)ws + planes);
        // A few slabs are summed inside the round/log pass (when its 16-byte accesses are legal); many
        // slabs of a small output go through a kernel of their own first, which has a thread per
        // output and more loads in flight (measured on the ResNet-50 weight gradients: summing 64 to
        // 256 slabs in the pass made those calls up to twice as long).
        const bool sum_in_pass = plan.splits <= 8 && (total % 2 == 0) && aligned(g.C32, 8) && (!g.C64 || aligned(g.C64, 16));
        double *reduced = sum_in_pass ? nullptr : partial + (uint64_t)plan.splits * total;
        void *ws_rl = (char *)partial + vt::gemm_split_bytes(M, N, batch, plan.splits);
        mark_begin(s);
        const hipError_t e2 = vt::launch_gemm_round_planes(g, plan, pl, partial, reduced, s);
        mark_end(s);
        if (e2 != hipSuccess) return VT_ERR_HIP;
        if (!sum_in_pass) return round_log_flat(reduced, total, g.thr, g.C32, log, ws_rl, s, /*mark=*/false);
        const vt::SplitKArgs a{partial, total, plan.splits, g.variant, g.alpha, g.bias, (uint32_t)N, g.C64};
        const uint32_t k = k_of(log->b_r);
        if (log->dense)
            return hip_status(vt::launch_splitk_log_dense(a, total, g.thr, k, g.C32, log->dense, log->count, (uint64_t *)ws_rl, s));
        return hip_status(vt::launch_splitk_log_onepass(a, total, g.thr, k, g.C32, ws_rl,
                                                        vt::LogOut{log->idx, log->dir, log->cap, log->count}, s));
    }
    const bool cleared = prepare_compaction(g, pl, log, total);
    g.tail_ws = (double *)((char *)ws + up256(planes));            // (the split-K slabs' place: free on this path)
    mark_begin(s);
    hipError_t e = vt::launch_gemm_round_planes(g, plan, pl, nullptr, nullptr, s);
    mark_end(s);
    if (e != hipSuccess) return VT_ERR_HIP;
    return finish_log(pl, (uint64_t)M * (uint64_t)batch, log, cleared, g.thr, s);
}

// Validates a convolution geometry and fills the internal descriptor (with the output size).
// Limits keep every index the kernel forms inside 32 bits.
bool conv_desc(const vt_conv2d *d, int64_t Cout, int mode, vt::ConvDesc *c)
{
    if (!d || Cout < 0 || (mode != VT_CONV_FORWARD && mode != VT_CONV_WEIGHT_GRAD && mode != VT_CONV_DATA_GRAD)) return false;
    const int64_t lim = (int64_t)1 << 24;
    if (d->N < 0 || d->H < 0 || d->W < 0 || d->C < 0 || d->KH < 1 || d->KW < 1 || d->stride_h < 1 || d->stride_w < 1 ||
        d->pad_h < 0 || d->pad_w < 0 || d->dil_h < 1 || d->dil_w < 1)
        return false;
    if (d->N >= lim || d->H >= lim || d->W >= lim || d->C >= lim || d->KH >= lim || d->KW >= lim || d->stride_h >= lim ||
        d->stride_w >= lim || d->pad_h >= lim || d->pad_w >= lim || d->dil_h >= lim || d->dil_w >= lim || Cout >= lim)
        return false;
    if (d->dil_h * (d->KH - 1) >= lim || d->dil_w * (d->KW - 1) >= lim) return false;
    const int64_t eh = d->H + 2 * d->pad_h - d->dil_h * (d->KH - 1) - 1;
    const int64_t ew = d->W + 2 * d->pad_w - d->dil_w * (d->KW - 1) - 1;
    c->N = d->N; c->H = d->H; c->W = d->W; c->C = d->C; c->KH = d->KH; c->KW = d->KW;
    c->stride_h = d->stride_h; c->stride_w = d->stride_w; c->pad_h = d->pad_h; c->pad_w = d->pad_w;
    c->dil_h = d->dil_h; c->dil_w = d->dil_w;
    c->Ho = eh < 0 ? 0 : eh / d->stride_h + 1;
    c->Wo = ew < 0 ? 0 : ew / d->stride_w + 1;
    const unsigned __int128 two31 = (unsigned __int128)1 << 31;
    if ((unsigned __int128)d->N * d->H * d->W * d->C >= two31) return false;          // image elements
    if ((unsigned __int128)d->N * c->Ho * c->Wo >= two31) return false;               // im2col rows
    if ((unsigned __int128)d->KH * d->KW * d->C >= two31) return false;               // taps
    if (mode == VT_CONV_DATA_GRAD) {                  // the gathered image is dY, the rows are input positions
        if ((unsigned __int128)d->N * c->Ho * c->Wo * Cout >= two31) return false;
        if ((unsigned __int128)d->N * d->H * d->W >= two31) return false;
        if ((unsigned __int128)d->KH * d->KW * Cout >= two31) return false;
        if (d->KH * d->KW > 65535) return false;      // one grid plane per filter position in the weight re-layout
    }
    return true;
}

// Input gradient of a convolution: dX (N H W x C) = view(dY) (N H W x KH KW Cout) times the filter
// re-laid as (KH KW Cout) x C.  The geometry is validated by the caller.
int conv_dgrad_entry(const vt::ConvDesc &c, int64_t Cout, const double *dY, const double *Wt, const double *bias,
                     float *C32, double *C64_debug, int variant, uint32_t thr, const vt_log *log, void *ws,
                     size_t ws_bytes, hipStream_t s)
{
    if (bias) return VT_ERR_INVALID_ARG;
    // (no output positions: dY is empty, nothing is read and the gradient is zero)
    const int64_t M = c.N * c.H * c.W, N = c.C, K = c.N * c.Ho * c.Wo == 0 ? 0 : c.KH * c.KW * Cout;
    if ((unsigned __int128)M * (unsigned __int128)N >= ((unsigned __int128)1 << 32)) return VT_ERR_INVALID_ARG;
    if (M * N == 0) {
        const vt::Planes pl = vt::planes_carve(ws, 0, 0);
        const vt::LogOut lo{log->idx, log->dir, log->cap, log->count};
        return hip_status(vt::launch_seg_scan(pl, lo, s));
    }
    if (!C32 || !aligned(C32, 4) || (C64_debug && !aligned(C64_debug, 8))) return VT_ERR_INVALID_ARG;
    if (K > 0 && (!dY || !Wt || !aligned(dY, 8) || !aligned(Wt, 8))) return VT_ERR_INVALID_ARG;
    vt::GemmArgs g;
    g.transA = 0; g.M = M; g.N = N; g.K = K; g.alpha = 1.0;
    g.A = dY; g.strideA = 0; g.strideB = 0;
    g.bias = nullptr; g.batch = 1; g.C32 = C32; g.ldc = N; g.strideC = 0;
    g.C64 = C64_debug; g.variant = variant; g.thr = thr;
    if (c.KH == 1 && c.KW == 1 && c.stride_h == 1 && c.stride_w == 1 && c.pad_h == 0 && c.pad_w == 0) {
        // a 1 x 1 filter at every position: dX = dY (rows x Cout) times the transposed filter (C x Cout
        // as it lies), a plain GEMM
        g.lda = Cout; g.B = Wt; g.transB = 1; g.ldb = Cout;
        return run_gemm(g, log, ws, ws_bytes, s);
    }
    const bool two_pass = k_of(log->b_r) != 0;
    const size_t at = dgrad_filter_offset(M, N, K, two_pass);
    if (!ws || !aligned(ws, 256) || ws_bytes < at + (size_t)K * (size_t)N * 8) return VT_ERR_WORKSPACE;
    double *Wp = (double *)((char *)ws + at);
    const uint64_t total = (uint64_t)M * (uint64_t)N;
    const bool phased = K > 0 && (c.stride_h > 1 || c.stride_w > 1) && c.stride_h <= 2 && c.stride_w <= 2 && N % 2 == 0 &&
                        aligned(C32, 8) && (!C64_debug || aligned(C64_debug, 16));
    if (phased) {
        // One GEMM per stride phase (no structural zeros multiplied), FP64 results side by side in
        // the workspace, then one round/log pass that looks every output up in its phase.
        double *slabs = (double *)((char *)ws + up256(round_log_bytes(total)));
        vt::PhaseArgs pa{};
        pa.P = slabs; pa.H = (uint32_t)c.H; pa.W = (uint32_t)c.W; pa.C = (uint32_t)c.C;
        pa.ph = (uint32_t)c.pad_h; pa.pw = (uint32_t)c.pad_w; pa.sh = (uint32_t)c.stride_h; pa.sw = (uint32_t)c.stride_w;
        pa.y64 = C64_debug;
        uint64_t slab_off = 0, w_off = 0;
        // the phases' GEMMs (different depths, each too small to fill the part) go out as one launch
        vt::GemmArgs group[4];
        vt::ConvDesc subs[4];
        double *outs[4];
        int count = 0;
        mark_begin(s);
        for (int64_t a = 0; a < c.stride_h; ++a)
            for (int64_t b = 0; b < c.stride_w; ++b) {
                const vt::PhaseAxis ax = vt::phase_axis(c.H, c.KH, c.stride_h, c.pad_h, c.dil_h, a);
                const vt::PhaseAxis bx = vt::phase_axis(c.W, c.KW, c.stride_w, c.pad_w, c.dil_w, b);
                const int idx = (int)(2 * a + b);
                pa.q0h[a] = (uint32_t)ax.q0; pa.Ha[a] = (uint32_t)ax.count;
                pa.q0w[b] = (uint32_t)bx.q0; pa.Wb[b] = (uint32_t)bx.count;
                pa.off[idx] = (uint32_t)slab_off;
                const int64_t rows = c.N * ax.count * bx.count, taps = ax.taps * bx.taps;
                if (rows == 0 || taps == 0) continue;            // no positions, or no filter tap reaches them: zeros
                pa.has |= 1u << idx;
                if (vt::launch_dgrad_weights(Wt, c.KW, c.C, Cout, ax.k0, ax.kstep, ax.taps, bx.k0, bx.kstep, bx.taps,
                                             Wp + w_off, s) != hipSuccess)
                    return VT_ERR_HIP;
                subs[count] = vt::ConvDesc{c.N, ax.count, bx.count, c.C, ax.taps, bx.taps, 1, 1, ax.pad, bx.pad, ax.dil, bx.dil, c.Ho, c.Wo};
                vt::GemmArgs &q = group[count];
                q = g;
                q.conv = &subs[count]; q.conv_dgrad_cout = Cout;
                q.M = rows; q.K = taps * Cout; q.lda = 0; q.B = Wp + w_off; q.transB = 0; q.ldb = N; q.raw = true;
                outs[count] = slabs + slab_off;
                ++count;
                slab_off += (uint64_t)rows * (uint64_t)N;
                w_off += (uint64_t)taps * (uint64_t)Cout * (uint64_t)N;
            }
        if (count) {
            // one tile shape for all: the one the plan takes for the phases together
            int64_t rows_all = 0, k_most = 0;
            for (int i = 0; i < count; ++i) { rows_all += group[i].M; k_most = group[i].K > k_most ? group[i].K : k_most; }
            const vt::GemmPlan plan = vt::plan_gemm(rows_all, N, k_most, 1, /*allow_split=*/false, vt::kALayoutRowMajor);
            if (vt::launch_gemm_group(group, outs, count, plan.shape, s) != hipSuccess) return VT_ERR_HIP;
        }
        mark_end(s);
        const uint32_t k = k_of(log->b_r);
        if (log->dense)
            return hip_status(vt::launch_phase_log_dense(pa, total, thr, k, C32, log->dense, log->count, (uint64_t *)ws, s));
        return hip_status(vt::launch_phase_log_onepass(pa, total, thr, k, C32, ws, vt::LogOut{log->idx, log->dir, log->cap, log->count}, s));
    }
    if (K > 0 && vt::launch_dgrad_weights(Wt, c.KW, c.C, Cout, 0, 1, c.KH, 0, 1, c.KW, Wp, s) != hipSuccess) return VT_ERR_HIP;
    g.conv = &c; g.conv_dgrad_cout = Cout;
    g.lda = 0; g.B = Wp; g.transB = 0; g.ldb = N;
    return run_gemm(g, log, ws, at, s);
}

}  // namespace

extern "C" {

uint32_t vt_thr_from_tau(double tau_ulp)
{
    if (!(tau_ulp >= 0.0 && tau_ulp <= 0.5)) return 0xFFFFFFFFu;
    return (uint32_t)std::ceil(std::ldexp(tau_ulp, 29));
}

uint32_t vt_thr_layer_from_stats(uint64_t thr_flip, uint64_t max_ulp64_diff)
{
    uint64_t need = thr_flip;
    if (max_ulp64_diff >= need) need = max_ulp64_diff == UINT64_MAX ? UINT64_MAX : max_ulp64_diff + 1;
    if (need >= VT_THR_LAYER_MAX) return VT_THR_LAYER_MAX;
    uint32_t thr = 1;
    while (thr < need) thr <<= 1;
    return thr;
}

const char *vt_strerror(int code)
{
    switch (code) {
    case VT_OK: return "ok";
    case VT_ERR_INVALID_ARG: return "invalid argument";
    case VT_ERR_WORKSPACE: return "workspace missing or too small";
    case VT_ERR_HIP: return "HIP call or kernel launch failed";
    case VT_ERR_UNSUPPORTED: return "unsupported request";
    case VT_ERR_STATIC_LIMIT: return "size beyond the limit of the library's static scratch";
    default: return "unknown status";
    }
}

size_t vt_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int64_t batch)
{
    (void)K;
    if (M < 0 || N < 0 || batch < 0) return 0;
    switch (op) {
    case VT_OP_ROUND_LOG: return round_log_bytes((uint64_t)M * (uint64_t)N * (uint64_t)batch);
    case VT_OP_LAYER_ROUND_LOG:
        return round_log_bytes((uint64_t)M * (uint64_t)N * (uint64_t)batch) + vt::layer_stat_bytes((uint64_t)M * (uint64_t)batch, (uint64_t)N);
    case VT_OP_GEMM_ROUND_LOG_BR:
        return vt::planes_bytes((uint64_t)M * (uint64_t)batch, (uint64_t)N) + vt::gemm_split_bytes(M, N, batch, max_splits(M, N, K, batch)) +
               round_log_bytes((uint64_t)M * (uint64_t)N * (uint64_t)batch);
    case VT_OP_GEMM_ROUND_LOG: {
        // sized for the split-K path too (taken for dense outputs when few tiles meet a long K)
        // ... and for the slices of tail tiles (the fused path)
        size_t bytes = up256(vt::planes_bytes((uint64_t)M * (uint64_t)batch, (uint64_t)N));
        const int splits = max_splits(M, N, K, batch);
        size_t extra = tail_bytes_for(M, N, K, batch);
        if (splits > 1) {
            const size_t sk = vt::gemm_split_bytes(M, N, batch, splits) + round_log_bytes((uint64_t)M * (uint64_t)N * (uint64_t)batch);
            extra = sk > extra ? sk : extra;
        }
        return bytes + extra;
    }
    case VT_OP_CONV_DGRAD_ROUND_LOG:
    case VT_OP_CONV_DGRAD_ROUND_LOG_BR: {
        // the GEMM's workspace, then the filter in the layout the GEMM multiplies by (K x N doubles)
        if (K < 0 || batch != 1) return 0;
        return dgrad_filter_offset(M, N, K, op == VT_OP_CONV_DGRAD_ROUND_LOG_BR) + (size_t)K * (size_t)N * 8;
    }
    case VT_OP_SHA256_TREE:
        if (K < 0 || (K % 64) != 0) return 0;
        return vt::sha256_tree_bytes((uint64_t)N, (uint64_t)K);
    case VT_OP_MERKLE_ROOT: return vt::merkle_root_bytes((uint64_t)N);
    default: return 0;
    }
}

int vt_sha256_tree(const void *data, uint64_t nbytes, uint64_t chunk, uint8_t *digest,
                   void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!digest || !aligned(digest, 4) || (chunk % 64) != 0) return VT_ERR_INVALID_ARG;
    if (nbytes && (!data || !aligned(data, 16))) return VT_ERR_INVALID_ARG;
    if (nbytes >= (1ull << 56)) return VT_ERR_INVALID_ARG;                       // chunk counts and bit lengths stay in range
    if (chunk == 0 && nbytes > (1ull << 26)) return VT_ERR_UNSUPPORTED;          // the sequential form is for small inputs
    if (chunk && nbytes / chunk >= (1ull << 36)) return VT_ERR_INVALID_ARG;      // grid limit: 2^31 workgroups of 64 chunks
    if (!ws || ws_bytes < vt::sha256_tree_bytes(nbytes, chunk) || !aligned(ws, 256)) return VT_ERR_WORKSPACE;
    return hip_status(vt::launch_sha256_tree((const uint8_t *)data, nbytes, chunk, (uint32_t *)digest, ws,
                                             (hipStream_t)hip_stream));
}

int vt_merkle_root(const uint8_t *leaves, uint64_t n_leaves, uint8_t *root, void *ws, size_t ws_bytes, void *hip_stream)
{
    if (!leaves || !root || n_leaves == 0 || !aligned(leaves, 4) || !aligned(root, 4)) return VT_ERR_INVALID_ARG;
    if (n_leaves >= (1ull << 36)) return VT_ERR_INVALID_ARG;
    if (!ws || ws_bytes < vt::merkle_root_bytes(n_leaves) || !aligned(ws, 256)) return VT_ERR_WORKSPACE;
    return hip_status(vt::launch_merkle_root((const uint32_t *)leaves, n_leaves, (uint32_t *)root, ws,
                                             (hipStream_t)hip_stream));
}

int vt_round_log(const double *x, uint64_t n, double tau_ulp, float *y, const vt_log *log,
                 void *ws, size_t ws_bytes, void *hip_stream)
{
    const uint32_t thr = vt_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || n >= (1ull << 32) || !log_ok(log)) return VT_ERR_INVALID_ARG;
    if (n && (!x || !y || !aligned(x, 8) || !aligned(y, 4))) return VT_ERR_INVALID_ARG;
    const size_t need = round_log_bytes(n);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return VT_ERR_WORKSPACE;
    return round_log_flat(x, n, thr, y, log, ws, (hipStream_t)hip_stream, /*mark=*/true);
}

int vt_round_log_static(const double *x, uint64_t n, double tau_ulp, float *y, const vt_log *log, void *hip_stream)
{
    const uint32_t thr = vt_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || !log_ok(log)) return VT_ERR_INVALID_ARG;
    if (n > VT_ROUND_LOG_STATIC_MAX_N) return VT_ERR_STATIC_LIMIT;
    if (n && (!x || !y || !aligned(x, 8) || !aligned(y, 4))) return VT_ERR_INVALID_ARG;
    // the sparse log's fallback for misaligned tensors needs bit-planes (n / 4 bytes): not held statically
    if (!log->dense && !vt::onepass_usable(x, y)) return VT_ERR_UNSUPPORTED;
    const size_t need = log->dense ? vt::dense_count_bytes() : vt::onepass_bytes(n);
    if (need > (size_t)VT_STATIC_SCRATCH_BYTES) return VT_ERR_STATIC_LIMIT;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != VT_OK) return rc;
    // (the kernels clear the words they use themselves, so the last call's contents do not matter)
    return round_log_flat(x, n, thr, y, log, ws, (hipStream_t)hip_stream, /*mark=*/true);
}

int vt_round_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                    uint64_t count, float *y, void *ws, size_t ws_bytes, void *hip_stream)
{
    (void)ws; (void)ws_bytes;
    return vt_round_replay_br(x, n, idx, dir, count, 32, y, hip_stream);
}

int vt_round_replay_br(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                       uint64_t count, int b_r, float *y, void *hip_stream)
{
    if (n >= (1ull << 32) || count >= (1ull << 32) || !br_ok(b_r)) return VT_ERR_INVALID_ARG;
    if (n && (!x || !y || !aligned(x, 8) || !aligned(y, 4))) return VT_ERR_INVALID_ARG;
    if (count && (!idx || !dir || !aligned(idx, 4) || !aligned(dir, 4))) return VT_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    mark_begin(s);
    const hipError_t e = vt::launch_replay(x, n, idx, dir, count, k_of(b_r), y, s);
    mark_end(s);
    return hip_status(e);
}

int vt_round_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, float *y, void *hip_stream)
{
    return vt_round_replay_dense_br(x, n, tlog, 32, y, hip_stream);
}

int vt_round_replay_dense_br(const double *x, uint64_t n, const uint8_t *tlog, int b_r, float *y, void *hip_stream)
{
    if (!br_ok(b_r)) return VT_ERR_INVALID_ARG;
    if (n && (!x || !y || !tlog || !aligned(x, 8) || !aligned(y, 4) || !aligned(tlog, 4))) return VT_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    mark_begin(s);
    const hipError_t e = vt::launch_replay_dense(x, n, tlog, k_of(b_r), y, s);
    mark_end(s);
    return hip_status(e);
}

// shared by the two GEMM entry points: batch_inner = 0 means one level of batching
static int gemm_entry(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                      const double *A, int64_t lda, int64_t strideA, const double *B, int64_t ldb, int64_t strideB,
                      const double *bias, int64_t batch, int64_t batch_inner, int64_t strideA_outer, int64_t strideB_outer,
                      float *C32, int64_t ldc, int64_t strideC, double *C64_debug, int variant,
                      double tau_ulp, const vt_log *log, void *ws, size_t ws_bytes, void *hip_stream)
{
    const uint32_t thr = vt_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || !log_ok(log)) return VT_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || batch < 0 || variant < 0 || variant > 1) return VT_ERR_INVALID_ARG;
    if ((transA != 0 && transA != 1) || (transB != 0 && transB != 1)) return VT_ERR_INVALID_ARG;
    if (batch_inner < 0 || strideA_outer < 0 || strideB_outer < 0) return VT_ERR_INVALID_ARG;
    if (batch_inner > 0 && batch % batch_inner != 0) return VT_ERR_INVALID_ARG;     // whole groups only
    if ((unsigned __int128)M * (unsigned __int128)N * (unsigned __int128)batch >= ((unsigned __int128)1 << 32))
        return VT_ERR_INVALID_ARG;          // log indices are 32-bit
    const uint64_t total = (uint64_t)M * (uint64_t)N * (uint64_t)batch;
    hipStream_t s = (hipStream_t)hip_stream;
    if (total == 0) {                       // nothing to compute; the log is empty
        const vt::Planes pl = vt::planes_carve(ws, 0, 0);
        const vt::LogOut lo{log->idx, log->dir, log->cap, log->count};
        return hip_status(vt::launch_seg_scan(pl, lo, s));
    }
    if (!C32 || !aligned(C32, 4) || ldc < N) return VT_ERR_INVALID_ARG;
    if (batch > 1) {                        // the matrices' outputs must not overlap: one after the other, or side by side
        const unsigned __int128 sc = strideC < 0 ? 0 : (unsigned __int128)strideC;
        const bool blocks = sc >= (unsigned __int128)(M - 1) * (unsigned __int128)ldc + (unsigned __int128)N;
        const bool columns = sc >= (unsigned __int128)N && (unsigned __int128)(batch - 1) * sc + (unsigned __int128)N <= (unsigned __int128)ldc;
        if (strideC < 0 || !(blocks || columns)) return VT_ERR_INVALID_ARG;
    }
    if (K > 0) {
        if (!A || !B || !aligned(A, 8) || !aligned(B, 8)) return VT_ERR_INVALID_ARG;
        if (lda < (transA ? M : K) || ldb < (transB ? K : N) || strideA < 0 || strideB < 0) return VT_ERR_INVALID_ARG;
    }
    if (C64_debug && !aligned(C64_debug, 8)) return VT_ERR_INVALID_ARG;
    vt::GemmArgs g;
    g.transA = transA; g.transB = transB; g.M = M; g.N = N; g.K = K; g.alpha = alpha;
    g.A = A; g.lda = lda; g.strideA = strideA; g.B = B; g.ldb = ldb; g.strideB = strideB;
    g.bias = bias; g.batch = batch; g.C32 = C32; g.ldc = ldc; g.strideC = strideC;
    g.batch_inner = batch_inner; g.strideA2 = strideA_outer; g.strideB2 = strideB_outer;
    g.C64 = C64_debug; g.variant = variant; g.thr = thr;
    return run_gemm(g, log, ws, ws_bytes, s);
}

int vt_gemm_f64_round_log(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                          const double *A, int64_t lda, int64_t strideA,
                          const double *B, int64_t ldb, int64_t strideB,
                          const double *bias, int64_t batch,
                          float *C32, int64_t ldc, int64_t strideC,
                          double *C64_debug, int variant,
                          double tau_ulp, const vt_log *log,
                          void *ws, size_t ws_bytes, void *hip_stream)
{
    return gemm_entry(transA, transB, M, N, K, alpha, A, lda, strideA, B, ldb, strideB, bias, batch, 0, 0, 0, C32, ldc,
                      strideC, C64_debug, variant, tau_ulp, log, ws, ws_bytes, hip_stream);
}

int vt_gemm_f64_round_log_nested(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                                 const double *A, int64_t lda, int64_t strideA, int64_t strideA_outer,
                                 const double *B, int64_t ldb, int64_t strideB, int64_t strideB_outer,
                                 const double *bias, int64_t batch_inner, int64_t batch_outer,
                                 float *C32, int64_t ldc, int64_t strideC,
                                 double *C64_debug, int variant,
                                 double tau_ulp, const vt_log *log,
                                 void *ws, size_t ws_bytes, void *hip_stream)
{
    if (batch_inner < 0 || batch_outer < 0) return VT_ERR_INVALID_ARG;
    if ((unsigned __int128)batch_inner * (unsigned __int128)batch_outer >= ((unsigned __int128)1 << 32)) return VT_ERR_INVALID_ARG;
    const int64_t batch = batch_inner * batch_outer;
    return gemm_entry(transA, transB, M, N, K, alpha, A, lda, strideA, B, ldb, strideB, bias, batch, batch_inner,
                      strideA_outer, strideB_outer, C32, ldc, strideC, C64_debug, variant, tau_ulp, log, ws, ws_bytes,
                      hip_stream);
}

int vt_conv2d_gemm_shape(const vt_conv2d *d, int64_t Cout, int mode, int64_t *M, int64_t *N, int64_t *K)
{
    vt::ConvDesc c;
    if (!M || !N || !K || !conv_desc(d, Cout, mode, &c)) return VT_ERR_INVALID_ARG;
    const int64_t rows = c.N * c.Ho * c.Wo, taps = c.KH * c.KW * c.C;
    if (mode == VT_CONV_DATA_GRAD) {
        *M = c.N * c.H * c.W;
        *N = c.C;
        *K = c.KH * c.KW * Cout;
        return VT_OK;
    }
    *M = mode == VT_CONV_FORWARD ? rows : taps;
    *N = Cout;
    *K = mode == VT_CONV_FORWARD ? taps : rows;
    return VT_OK;
}

int vt_conv2d_f64_round_log(int mode, const vt_conv2d *d, int64_t Cout, const double *X, const double *B,
                            const double *bias, float *C32, double *C64_debug, int variant,
                            double tau_ulp, const vt_log *log, void *ws, size_t ws_bytes, void *hip_stream)
{
    const uint32_t thr = vt_thr_from_tau(tau_ulp);
    vt::ConvDesc c;
    if (thr == 0xFFFFFFFFu || !log_ok(log) || variant < 0 || variant > 1) return VT_ERR_INVALID_ARG;
    if (!conv_desc(d, Cout, mode, &c)) return VT_ERR_INVALID_ARG;
    if (mode == VT_CONV_WEIGHT_GRAD && bias) return VT_ERR_INVALID_ARG;
    const int64_t rows = c.N * c.Ho * c.Wo, taps = c.KH * c.KW * c.C;
    if (mode == VT_CONV_DATA_GRAD)
        return conv_dgrad_entry(c, Cout, X, B, bias, C32, C64_debug, variant, thr, log, ws, ws_bytes, (hipStream_t)hip_stream);
    const int64_t M = mode == VT_CONV_FORWARD ? rows : taps, K = mode == VT_CONV_FORWARD ? taps : rows;
    if ((unsigned __int128)M * (unsigned __int128)Cout >= ((unsigned __int128)1 << 32)) return VT_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)hip_stream;
    if (M * Cout == 0) {
        const vt::Planes pl = vt::planes_carve(ws, 0, 0);
        const vt::LogOut lo{log->idx, log->dir, log->cap, log->count};
        return hip_status(vt::launch_seg_scan(pl, lo, s));
    }
    if (!C32 || !aligned(C32, 4) || (C64_debug && !aligned(C64_debug, 8))) return VT_ERR_INVALID_ARG;
    if (K > 0 && (!X || !B || !aligned(X, 8) || !aligned(B, 8))) return VT_ERR_INVALID_ARG;
    vt::GemmArgs g;
    g.conv = &c; g.conv_wgrad = mode == VT_CONV_WEIGHT_GRAD;
    g.transA = g.conv_wgrad ? 1 : 0; g.transB = 0; g.M = M; g.N = Cout; g.K = K; g.alpha = 1.0;
    g.A = X; g.lda = 0; g.strideA = 0; g.B = B; g.ldb = Cout; g.strideB = 0;
    g.bias = bias; g.batch = 1; g.C32 = C32; g.ldc = Cout; g.strideC = 0;
    g.C64 = C64_debug; g.variant = variant; g.thr = thr;
    if (c.KH == 1 && c.KW == 1 && c.stride_h == 1 && c.stride_w == 1 && c.pad_h == 0 && c.pad_w == 0) {
        // a 1 x 1 filter at every position: the im2col matrix is the image itself, rows (n, h, w) by
        // channels, so the plain operand loader (no address arithmetic in the loop) reads it as it lies
        g.conv = nullptr;
        g.lda = c.C;
    }
    return run_gemm(g, log, ws, ws_bytes, s);
}

int vt_layer_f64_round_log(const vt_layer *L, float *y, double *y64_debug, int variant,
                           double tau_ulp, const vt_log *log, void *ws, size_t ws_bytes, void *hip_stream)
{
    const uint32_t thr = vt_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || !log_ok(log) || !L || variant < 0 || variant > 1) return VT_ERR_INVALID_ARG;
    if (L->op < VT_LAYER_ADD || L->op > VT_LAYER_BATCHNORM_RELU || L->rows < 0 || L->cols < 0 || L->causal_period < 0)
        return VT_ERR_INVALID_ARG;
    if ((unsigned __int128)L->rows * (unsigned __int128)L->cols >= ((unsigned __int128)1 << 32)) return VT_ERR_INVALID_ARG;
    if (L->causal_period >= ((int64_t)1 << 32)) return VT_ERR_INVALID_ARG;
    const uint64_t n = (uint64_t)L->rows * (uint64_t)L->cols;
    if (n) {
        if (!L->a || !y || !aligned(L->a, 16) || !aligned(y, 8)) return VT_ERR_INVALID_ARG;
        if (L->op == VT_LAYER_ADD && (!L->b || !aligned(L->b, 16))) return VT_ERR_INVALID_ARG;
        if ((L->gamma && !aligned(L->gamma, 8)) || (L->beta && !aligned(L->beta, 8))) return VT_ERR_INVALID_ARG;
        if (y64_debug && !aligned(y64_debug, 16)) return VT_ERR_INVALID_ARG;
        if ((L->op == VT_LAYER_NORM || L->op >= VT_LAYER_BATCHNORM) && !(L->eps >= 0.0)) return VT_ERR_INVALID_ARG;
    }
    const size_t rl = round_log_bytes(n);
    if (!ws || ws_bytes < rl + vt::layer_stat_bytes((uint64_t)L->rows, (uint64_t)L->cols) || !aligned(ws, 256))
        return VT_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)hip_stream;
    vt::LayerArgs g;
    g.op = L->op; g.a = L->a; g.b = L->b;
    const bool affine = L->op == VT_LAYER_NORM || L->op >= VT_LAYER_BATCHNORM;
    g.gamma = affine ? L->gamma : nullptr;
    g.beta = affine ? L->beta : nullptr;
    g.stat = (const double *)((char *)ws + rl);
    g.y64 = y64_debug;
    g.cols = (uint32_t)(L->cols > 0 ? L->cols : 1);
    g.inv_cols = 1.0 / (double)g.cols;
    g.scale = L->scale;
    g.period = L->op == VT_LAYER_SOFTMAX ? (uint32_t)L->causal_period : 0u;
    g.inv_period = g.period ? 1.0 / (double)g.period : 0.0;
    g.eps = L->eps;
    g.variant = variant;
    const bool rowwise = n && vt::rowwise_usable(L->op, (uint64_t)L->cols) &&
                         vt::rowwise_bytes((uint64_t)L->rows) <= rl;
    hipError_t e = rowwise ? hipSuccess : vt::launch_layer_stats(g, (uint64_t)L->rows, s);
    if (e != hipSuccess) return VT_ERR_HIP;
    const uint32_t k = k_of(log->b_r);
    if (rowwise) {                          // a row at a time in registers: no statistics pass before it
        mark_begin(s);
        if (log->dense) e = vt::launch_rowwise_dense(g, (uint64_t)L->rows, thr, k, y, log->dense, log->count, (uint64_t *)ws, s);
        else e = vt::launch_rowwise_onepass(g, (uint64_t)L->rows, thr, k, y, ws, vt::LogOut{log->idx, log->dir, log->cap, log->count}, s);
        mark_end(s);
        return hip_status(e);
    }
    mark_begin(s);
    if (log->dense) e = vt::launch_layer_log_dense(g, n, thr, k, y, log->dense, log->count, (uint64_t *)ws, s);
    else e = vt::launch_layer_log_onepass(g, n, thr, k, y, ws, vt::LogOut{log->idx, log->dir, log->cap, log->count}, s);
    mark_end(s);
    return hip_status(e);
}

int vt_threshold_stats(const double *y1, const double *y2, uint64_t n, uint64_t *out, void *hip_stream)
{
    return vt_threshold_stats_br(y1, y2, n, 32, out, hip_stream);
}

int vt_threshold_stats_br(const double *y1, const double *y2, uint64_t n, int b_r, uint64_t *out, void *hip_stream)
{
    if (!out || !aligned(out, 8) || !br_ok(b_r)) return VT_ERR_INVALID_ARG;
    if (n && (!y1 || !y2 || !aligned(y1, 8) || !aligned(y2, 8))) return VT_ERR_INVALID_ARG;
    return hip_status(vt::launch_stats(y1, y2, n, k_of(b_r), out, (hipStream_t)hip_stream));
}

int vt_gemm_plan(int transA, int64_t M, int64_t N, int64_t K, int64_t batch, int64_t ldc, int64_t strideC,
                 int *tile_m, int *tile_n, int *splits)
{
    if (M < 0 || N < 0 || K < 0 || batch < 0 || !tile_m || !tile_n || !splits) return VT_ERR_INVALID_ARG;
    if (transA != VT_A_ROW_MAJOR && transA != VT_A_TRANSPOSED && transA != VT_A_IM2COL_T) return VT_ERR_INVALID_ARG;
    const vt::GemmPlan plan = vt::plan_gemm(M, N, K, batch, split_allowed(M, N, batch, ldc, strideC), transA);
    static const int bm[2] = {128, 64}, bn[2] = {128, 64};
    *tile_m = bm[plan.shape];
    *tile_n = bn[plan.shape];
    *splits = plan.splits;
    return VT_OK;
}

int vt_gemm_tail_plan(int transA, int64_t M, int64_t N, int64_t K, int64_t batch, int64_t ldc, int64_t strideC,
                      int *tail_tiles, int *slices)
{
    int tm, tn, splits;
    if (!tail_tiles || !slices) return VT_ERR_INVALID_ARG;
    const int rc = vt_gemm_plan(transA, M, N, K, batch, ldc, strideC, &tm, &tn, &splits);
    if (rc != VT_OK) return rc;
    *tail_tiles = 0;
    *slices = 1;
    if (splits != 1 || M == 0 || N == 0 || batch == 0) return VT_OK;
    const uint64_t tiles = (uint64_t)((M + tm - 1) / tm) * (uint64_t)((N + tn - 1) / tn) * (uint64_t)batch;
    if (vt::gemm_tail_cut(tm == 128 ? 0 : 1, tiles, (K + 15) / 16)) {
        *tail_tiles = (int)(tiles % 256u);
        *slices = 4;
    }
    return VT_OK;
}

int vt_set_kernel_events(void *ev_begin, void *ev_end)
{
    if ((ev_begin == nullptr) != (ev_end == nullptr)) return VT_ERR_INVALID_ARG;
    g_ev_begin = (hipEvent_t)ev_begin;
    g_ev_end = (hipEvent_t)ev_end;
    return VT_OK;
}

}  // extern "C"
