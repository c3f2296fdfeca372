// vt_gemm_kernels.hip -- FP64 MFMA GEMM with the trainer hook fused into its epilogue (gfx950).
//
// C64 = alpha * op(A) op(B) (+ bias) is accumulated with v_mfma_f64_16x16x4_f64; each
// accumulator element is rounded to FP32, tested against the logging threshold and its
// decision written as one bit of two row-major bit-planes, all from registers: the FP64
// result never goes to memory (unless the caller asks for the debug copy).
//
// Tiling: a workgroup is 256 threads = 4 waves arranged WM x WN (2 x 2 or 4 x 1); a wave owns
// TM x 4 MFMA tiles of 16 x 16, i.e. 16 TM rows by 64 columns, so that one wave always produces
// whole 64-bit words of the decision planes.  Workgroup tiles: 128 x 128 (2x2, TM 4: the large
// shape, 128 accumulator registers per lane, two workgroups per CU) and 64 x 64 (4x1, TM 1: four
// workgroups per CU) for narrow outputs, short K and problems with too few large tiles to fill
// 256 CUs; the host plan picks one per problem.
// K step 16; operands are staged through LDS in k-major order ([k][m], [k][n]), double-buffered
// against the global loads, and the next tile is written to LDS in the shadow of the last MFMA
// group of the current one.
//
// Split-K (weight-gradient shapes: tiny outputs, very long K): the K range is cut into `splits`
// contiguous slices, every slice writes its raw FP64 accumulators to its own workspace slab, and
// a second kernel adds the slabs in a fixed order before the single rounding -- the order of
// additions never depends on timing.
//
// Lane layout of v_mfma_f64_16x16x4_f64 (measured on gfx950):
//   A operand: lane l holds A[i = l % 16][k = l / 16];  B operand: lane l holds B[k = l / 16][j = l % 16]
//   D: register r of lane l holds D[i = 4 r + l / 16][j = l % 16].
// This file: the tile-shape and split-K plan, the split-K reduction and the launcher; the kernel
// template lives in vt_gemm_tile.h.
#include "vt_gemm_tile.h"

#include <cmath>
#include <cstdlib>

namespace vt {

namespace {

// Split-K second stage: out[e] = alpha * (P[0][e] + P[1][e] + ...) (+ bias[col]), slabs added in
// ascending order (variant 0) or descending order (variant 1).  One thread per output.
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const double *__restrict__ P, uint64_t slab, int splits,
                                                            int variant, double alpha, const double *__restrict__ bias,
                                                            uint32_t N, double *__restrict__ out,
                                                            double *__restrict__ out2)
{
    const uint64_t e = (uint64_t)blockIdx.x * 256u + threadIdx.x;
    if (e >= slab) return;
    double s = 0.0;
    int k = 0;
    for (; k + 8 <= splits; k += 8) {                      // eight loads in flight, additions still in order
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = P[(uint64_t)(variant ? splits - 1 - (k + u) : k + u) * slab + e];
#pragma unroll
        for (int u = 0; u < 8; ++u) s = s + v[u];
    }
    for (; k < splits; ++k) s = s + P[(uint64_t)(variant ? splits - 1 - k : k) * slab + e];
    double c = alpha * s;
    if (bias) c = c + bias[e % N];
    out[e] = c;
    if (out2) out2[e] = c;
}

// bm x bn, measured MFMA efficiency with a full CU, workgroups that fit on one CU (LDS-bound),
// cost of a tile's start and epilogue in k steps
struct TileShape { int wm, tm, bm, bn; double eff; int conc; double overhead; };
constexpr int kNumShapes = 2;
constexpr TileShape kShapes[kNumShapes] = {{2, 4, 128, 128, 0.928, 2, 6.0}, {4, 1, 64, 64, 0.891, 4, 5.6}};
// the same for an A operand stored transposed (its tiles go into LDS as they lie, the other
// operand's pattern) ...
constexpr TileShape kShapesT[kNumShapes] = {{2, 4, 128, 128, 0.72, 2, 9.7}, {4, 1, 64, 64, 0.809, 4, 5.3}};
// ... and for the transposed implicit-im2col view of a convolution's weight gradient, whose gather
// costs the small tile more than the large one
constexpr TileShape kShapesG[kNumShapes] = {{2, 4, 128, 128, 0.82, 2, 9.7}, {4, 1, 64, 64, 0.641, 4, 4.9}};

constexpr uint32_t kTailTilesMax = 64;

}  // namespace

// Tail tiles.  All tiles of a launch take equally long and the compute units take them in turn, so
// a launch of 256 f + r tiles runs as long as one of 256 (f + 1).  When r <= 64, the last r tiles are
// cut along k into four slices each -- at most 256 short workgroups, a quarter tile time -- and a
// small kernel adds the slices in a fixed order and applies the epilogue.  (Larger r, where the
// slices take two or three quarters, measured no gain.)  True when the tail is cut: when the time
// saved (from measured per-step costs of the two tiles) exceeds the small kernel's 6 us twice over --
// thresholds of 20 / 12 / 7 us gave 9.85 / 9.64 / 9.73 ms on the ResNet-50 forward stream; slices
// shorter than eight k steps (K < 512) are mostly prologue and lost.  A pure function of the shape,
// like the plan.
bool gemm_tail_cut(int shape, uint64_t tiles, int64_t nkt)
{
    const uint64_t full = tiles / 256u, rem = tiles % 256u;
    if (full < 1 || full > 16 || rem < 1 || rem > kTailTilesMax || nkt < 32) return false;
    const double tile_us = shape == 0 ? ((double)nkt + 6.0) * 1.9 : ((double)nkt + 5.6) * 0.47;
    return tile_us * 0.75 >= 12.0;
}

// Tile shape and split count for a problem, from a small cost model calibrated on the box (unit:
// a quarter MFMA-pipe cycle per CU): rounds of 256 workgroups x work per workgroup / efficiency
// of the shape (lower when the grid leaves resident slots of a CU empty, so that stalls are not
// hidden), plus
// for split-K the two extra kernels and the slab traffic.  Pure host arithmetic on the shape, so
// the choice (and with it the accumulation order) is a function of the arguments alone.
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int64_t batch, bool allow_split, int a_layout)
{
    GemmPlan best{0, 1, 0};
    double best_cost = 1e300;
    const int64_t nkt = (K + BK - 1) / BK;
    for (int sh = 0; sh < kNumShapes; ++sh) {
        const TileShape &t = a_layout == kALayoutIm2colT ? kShapesG[sh] : (a_layout == kALayoutTransposed ? kShapesT[sh] : kShapes[sh]);
        const double tiles = (double)((M + t.bm - 1) / t.bm) * (double)((N + t.bn - 1) / t.bn) * (double)batch;
        // split factors: every count up to 16 (so that tiles x slices can fill whole rounds), then coarser
        static const int kSplits[] = {1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 20, 24, 28, 32, 40, 48, 56, 64, 80, 96,
                                      112, 128, 160, 192, 224, 256};
        for (int sp : kSplits) {
            if (sp > 1 && (!allow_split || nkt / sp < 8)) break;        // keep >= 8 k steps per slice
            const double blocks = tiles * sp;
            double rounds = std::ceil(blocks / 256.0);
            const double eff = t.eff * (rounds >= (double)t.conc ? 1.0 : 0.782);
            // (the fused path shares its last few tiles among several workgroups: a fraction of a round, and a small kernel)
            const bool tail = sp == 1 && gemm_tail_cut(sh, (uint64_t)tiles, nkt);
            if (tail) rounds = std::floor(blocks / 256.0) + 0.25;
            double cost = rounds * (double)t.bm * t.bn * ((double)((nkt + sp - 1) / sp) + t.overhead) / eff;
            if (tail) cost += 40000.0;
            if (sp > 1) cost += 173000.0 + 0.0171 * (double)M * N * batch * (sp + 2);
            if (cost < best_cost) { best_cost = cost; best = GemmPlan{sh, sp, 0}; }
        }
    }
    best.kt_per_split = (int)((nkt + best.splits - 1) / best.splits);
    if (best.kt_per_split < 1) best.kt_per_split = 1;
    return best;
}

size_t gemm_split_bytes(int64_t M, int64_t N, int64_t batch, int splits)
{
    if (splits < 1) return 0;
    const uint64_t slab = (uint64_t)M * N * batch * 8;
    return (size_t)((slab + 255) / 256 * 256 * (uint64_t)(splits + 1));   // slabs + the reduced tensor
}

namespace {

// one 32 x 32 block of one filter position, transposed through LDS (reads and writes coalesced)
__global__ __launch_bounds__(256) void dgrad_weights_kernel(const double *__restrict__ Wt, uint32_t KW, uint32_t C, uint32_t Cout,
                                                            uint32_t kh0, uint32_t sth, uint32_t kw0, uint32_t stw, uint32_t nkw,
                                                            double *__restrict__ Wp)
{
    __shared__ double tile[32][33];
    const uint32_t tx = threadIdx.x & 31u, ty = threadIdx.x >> 5;            // 32 x 8 threads
    const uint32_t ih = blockIdx.z / nkw, iw = blockIdx.z % nkw;
    const uint64_t plane = (uint64_t)C * Cout;
    const uint64_t src = (uint64_t)((kh0 + sth * ih) * KW + kw0 + stw * iw) * plane, dst = (uint64_t)blockIdx.z * plane;
    const uint32_t co0 = blockIdx.x * 32u, c0 = blockIdx.y * 32u;
#pragma unroll
    for (uint32_t i = 0; i < 32; i += 8) {
        const uint32_t c = c0 + ty + i, co = co0 + tx;
        if (c < C && co < Cout) tile[ty + i][tx] = Wt[src + (uint64_t)c * Cout + co];
    }
    __syncthreads();
#pragma unroll
    for (uint32_t i = 0; i < 32; i += 8) {
        const uint32_t co = co0 + ty + i, c = c0 + tx;
        if (c < C && co < Cout) Wp[dst + (uint64_t)co * C + c] = tile[tx][ty + i];
    }
}

}  // namespace

hipError_t launch_dgrad_weights(const double *Wt, int64_t KW, int64_t C, int64_t Cout, int64_t kh0, int64_t sth, int64_t nkh,
                                int64_t kw0, int64_t stw, int64_t nkw, double *Wp, hipStream_t s)
{
    if (nkh <= 0 || nkw <= 0 || C <= 0 || Cout <= 0) return hipSuccess;
    const uint64_t gx = (uint64_t)(Cout + 31) / 32, gy = (uint64_t)(C + 31) / 32, gz = (uint64_t)nkh * (uint64_t)nkw;
    if (gx > 0x7FFFFFFFull || gy > 65535ull || gz > 65535ull) return hipErrorInvalidValue;
    dgrad_weights_kernel<<<dim3((uint32_t)gx, (uint32_t)gy, (uint32_t)gz), 256, 0, s>>>(
        Wt, (uint32_t)KW, (uint32_t)C, (uint32_t)Cout, (uint32_t)kh0, (uint32_t)sth, (uint32_t)kw0, (uint32_t)stw, (uint32_t)nkw, Wp);
    return hipGetLastError();
}

namespace {

// Kernel parameters of one problem (am, kcb: the kernel's operand modes).  total_blocks = 0: nothing to launch.
hipError_t build_params(const GemmArgs &g, const GemmPlan &plan, const Planes &pl, double *partial, GemmParams &p, int &am,
                        bool &kcb)
{
    const TileShape &t = kShapes[plan.shape];
    p.A = g.A; p.B = g.B; p.bias = g.bias; p.C32 = g.C32; p.C64 = g.C64; p.partial = partial;
    p.pl_logged = pl.logged; p.pl_dir = pl.dir;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.strideA = g.strideA; p.strideB = g.strideB; p.strideC = g.strideC; p.batch = g.batch;
    p.batch_inner = (uint32_t)(g.batch_inner > 0 ? g.batch_inner : (g.batch > 0 ? g.batch : 1));
    p.strideA2 = g.strideA2; p.strideB2 = g.strideB2;
    p.alpha = g.alpha; p.thr = g.thr; p.wpr = pl.wpr; p.variant = g.variant;
    p.splits = plan.splits; p.kt_per_split = plan.kt_per_split; p.raw = g.raw ? 1 : 0;
    p.tilesM = (uint32_t)((g.M + t.bm - 1) / t.bm);
    p.tilesN = (uint32_t)((g.N + t.bn - 1) / t.bn);
    const uint64_t per_split = (uint64_t)p.tilesM * p.tilesN * (uint64_t)g.batch;
    const uint64_t total = per_split * (uint64_t)plan.splits;
    if (total > 0x7FFFFFFFull) return hipErrorInvalidValue;
    p.tiles_per_split = (uint32_t)per_split;
    p.total_blocks = (uint32_t)total;
    p.tiles_total = (uint32_t)total;
    p.tail_first = p.tiles_total; p.tail_shift = 0; p.tail_kt = 0; p.tail_partial = nullptr;
    if (g.tail_ws && plan.splits == 1 && !g.raw) {      // tail tiles (gemm_tail_quarters)
        const int64_t nkt = (g.K + BK - 1) / BK;
        if (gemm_tail_cut(plan.shape, p.tiles_total, nkt)) {
            const uint32_t rem = p.tiles_total % 256u, shift = 2;
            p.tail_first = p.tiles_total - rem;
            p.tail_shift = shift;
            p.tail_kt = (uint32_t)((nkt + (1 << shift) - 1) >> shift);
            p.tail_partial = g.tail_ws;
            p.total_blocks = p.tail_first + (rem << shift);
        }
    }
    p.m_tiles_per_split = magic_of(p.tiles_per_split);
    p.m_per_batch = magic_of(p.tilesM * p.tilesN);
    p.m_width = magic_of(8u * p.tilesN);
    p.m_batch_inner = magic_of(p.batch_inner);
    p.zero_a = g.zero_a; p.zero_a_words = g.zero_a_words; p.zero_b = g.zero_b; p.zero_b_words = g.zero_b_words;
    p.vecA = ((uintptr_t)g.A % 16 == 0) && (g.lda % 2 == 0) && (g.strideA % 2 == 0) && (g.strideA2 % 2 == 0);
    p.vecB = ((uintptr_t)g.B % 16 == 0) && (g.ldb % 2 == 0) && (g.strideB % 2 == 0) && (g.strideB2 % 2 == 0);
    kcb = g.transB != 0;
    am = g.transA ? 0 : 1;
    p.conv = ConvGeom{};
    if (g.conv) {
        // A is the image; the matrix the kernel multiplies is its im2col view (transposed for the
        // weight gradient).  The caller has checked the geometry (sizes below 2^31).
        const ConvDesc &d = *g.conv;
        p.conv = conv_geom(d.N, d.H, d.W, d.C, d.KH, d.KW, d.stride_h, d.stride_w, d.pad_h, d.pad_w, d.dil_h, d.dil_w,
                           d.Ho, d.Wo, (d.C % 2 == 0) && ((uintptr_t)g.A % 16 == 0));
        am = g.conv_wgrad ? 3 : 2;
        if (g.conv_dgrad_cout > 0) {
            p.conv = dgrad_geom(d.N, d.H, d.W, g.conv_dgrad_cout, d.KH, d.KW, d.stride_h, d.stride_w, d.pad_h, d.pad_w,
                                d.dil_h, d.dil_w, d.Ho, d.Wo, (g.conv_dgrad_cout % 2 == 0) && ((uintptr_t)g.A % 16 == 0));
            am = 4;
        }
        p.vecA = p.conv.vec;
    }
    return hipSuccess;
}

}  // namespace

hipError_t launch_gemm_round_planes(const GemmArgs &g, const GemmPlan &plan, const Planes &pl, double *partial,
                                    double *reduced, hipStream_t s)
{
    GemmParams p;
    int am;
    bool kcb;
    hipError_t e = build_params(g, plan, pl, partial, p, am, kcb);
    if (e != hipSuccess || p.total_blocks == 0) return e;
    switch (plan.shape) {
    case 0: e = launch_gemm_128x128(p, am, kcb, s); break;
    default: e = launch_gemm_64x64(p, am, kcb, s); break;
    }
    if (e != hipSuccess || (plan.splits <= 1 && !g.raw) || !reduced) return e;     // no `reduced`: the caller sums the slabs itself
    const uint64_t slab = (uint64_t)g.M * g.N * g.batch;
    splitk_reduce_kernel<<<(uint32_t)((slab + 255) / 256), 256, 0, s>>>(partial, slab, plan.splits, g.variant, g.alpha,
                                                                      g.bias, (uint32_t)g.N, reduced, g.C64);
    return hipGetLastError();
}

// Up to kGroupMax problems (raw accumulators to partial[i], no planes) of one tile shape in one launch.
hipError_t launch_gemm_group(const GemmArgs *g, double *const *partial, int count, int shape, hipStream_t s)
{
    if (count < 1 || count > kGroupMax) return hipErrorInvalidValue;
    GemmGroup gp{};
    GemmPlan plan{shape, 1, 0};
    int am0 = -1;
    bool kcb0 = false;
    uint32_t at = 0;
    for (int i = 0; i < kGroupMax; ++i) {
        gp.first[i] = at;
        if (i >= count) { gp.p[i] = gp.p[0]; continue; }
        plan.kt_per_split = (int)((g[i].K + BK - 1) / BK);
        if (plan.kt_per_split < 1) plan.kt_per_split = 1;
        int am;
        bool kcb;
        const hipError_t e = build_params(g[i], plan, Planes{}, partial[i], gp.p[i], am, kcb);
        if (e != hipSuccess) return e;
        if (i == 0) { am0 = am; kcb0 = kcb; }
        else if (am != am0 || kcb != kcb0) return hipErrorInvalidValue;
        if ((uint64_t)at + gp.p[i].total_blocks > 0x7FFFFFFFull) return hipErrorInvalidValue;
        at += gp.p[i].total_blocks;
    }
    gp.first[kGroupMax] = at;
    if (at == 0) return hipSuccess;
    return shape == 0 ? launch_gemm_grouped_128x128(gp, am0, kcb0, s) : launch_gemm_grouped_64x64(gp, am0, kcb0, s);
}

}  // namespace vt
