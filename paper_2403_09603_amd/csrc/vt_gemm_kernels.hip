// vt_gemm_kernels.hip -- FP64 MFMA GEMM with the trainer hook fused into its epilogue (gfx950).
//
// C64 = alpha * op(A) op(B) (+ bias) is accumulated with v_mfma_f64_16x16x4_f64; each
// accumulator element is rounded to FP32, tested against the logging threshold and its
// decision written as one bit of two row-major bit-planes, all from registers: the FP64
// result never goes to memory (unless the caller asks for the debug copy).
//
// Tiling: workgroup 256 threads = 2 x 2 waves, workgroup tile 128 x 128, wave tile 64 x 64 =
// 4 x 4 MFMA tiles (128 accumulator registers per lane), K step 16, operands staged through
// LDS in k-major order ([k][m], [k][n]) and double-buffered against the global loads.
//
// Lane layout of v_mfma_f64_16x16x4_f64 (measured on gfx950):
//   A operand: lane l holds A[i = l % 16][k = l / 16];  B operand: lane l holds B[k = l / 16][j = l % 16]
//   D: register r of lane l holds D[i = 4 r + l / 16][j = l % 16].
#include "vt_device.h"
#include "vt_kernels.h"

namespace vt {

namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));

constexpr int BM = 128, BN = 128, BK = 16;
constexpr int LDS_S = 128 + 16;                 // row pitch in doubles: k rows 32 banks apart
constexpr int kTileDoubles = BK * LDS_S;

struct GemmParams {
    const double *A, *B, *bias;
    float *C32;
    double *C64;
    uint64_t *pl_logged, *pl_dir;
    int64_t M, N, K, lda, ldb, ldc, strideA, strideB, strideC;
    double alpha;
    uint32_t thr, wpr, tilesM, tilesN, total_tiles;
    int variant, vecA, vecB;
};

// Global -> registers for one 128 x 16 operand tile.  KC = the operand is contiguous along k
// (element (mn, k) at base[mn * ld + k]); otherwise contiguous along m/n (base[k * ld + mn]).
// Out-of-range elements read as 0, so partial tiles add exact zeros.
template <bool KC>
__device__ __forceinline__ void load_tile(const double *__restrict__ base, int64_t ld, int64_t mn0, int64_t k0,
                                          int64_t MN, int64_t K, int vec, d2 (&regs)[4])
{
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        int64_t mn, k;
        if (KC) { mn = mn0 + (t >> 3) + 32 * j; k = k0 + (t & 7) * 2; }
        else    { k = k0 + (t >> 6) + 4 * j;    mn = mn0 + (t & 63) * 2; }
        d2 v = {0.0, 0.0};
        if (KC) {
            if (mn < MN) {
                const double *p = base + mn * ld + k;
                if (vec && k + 1 < K) v = *(const d2 *)p;
                else { if (k < K) v.x = p[0]; if (k + 1 < K) v.y = p[1]; }
            }
        } else {
            if (k < K) {
                const double *p = base + k * ld + mn;
                if (vec && mn + 1 < MN) v = *(const d2 *)p;
                else { if (mn < MN) v.x = p[0]; if (mn + 1 < MN) v.y = p[1]; }
            }
        }
        regs[j] = v;
    }
}

// Same tile when it lies wholly inside the operand and 16-byte loads are legal: four straight
// vector loads from a per-thread pointer to the tile's k = 0 position, no guards.
template <bool KC>
__device__ __forceinline__ const double *tile_origin(const double *__restrict__ base, int64_t ld, int64_t mn0)
{
    const int t = threadIdx.x;
    return KC ? base + (mn0 + (t >> 3)) * ld + (t & 7) * 2 : base + (int64_t)(t >> 6) * ld + mn0 + (t & 63) * 2;
}

template <bool KC>
__device__ __forceinline__ void load_tile_fast(const double *__restrict__ origin, int64_t ld, int64_t k0, d2 (&regs)[4])
{
    const double *p = KC ? origin + k0 : origin + k0 * ld;
    const int64_t step = KC ? 32 * ld : 4 * ld;
#pragma unroll
    for (int j = 0; j < 4; ++j) regs[j] = *(const d2 *)(p + j * step);
}

template <bool KC>
__device__ __forceinline__ void store_tile(double *__restrict__ S, const d2 (&regs)[4])
{
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (KC) {
            const int mn = (t >> 3) + 32 * j, k = (t & 7) * 2;
            S[k * LDS_S + mn] = regs[j].x;
            S[(k + 1) * LDS_S + mn] = regs[j].y;
        } else {
            const int k = (t >> 6) + 4 * j, mn = (t & 63) * 2;
            *(d2 *)&S[k * LDS_S + mn] = regs[j];
        }
    }
}

template <bool KCA, bool KCB>
__global__ __launch_bounds__(256, 2) void gemm_round_planes_kernel(const GemmParams p)
{
    __shared__ double lds[4 * kTileDoubles];     // A0 A1 B0 B1
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv >> 1, wn = wv & 1;

    // Workgroup -> tile.  Consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2), so ids are first regrouped per XCD, then walked in bands of 8 row
    // tiles so that neighbours in time share A and B panels in that L2.
    uint32_t pid;
    {
        const uint32_t i = blockIdx.x, q = p.total_tiles / 8u, r = p.total_tiles % 8u, xcd = i % 8u;
        pid = xcd * q + (xcd < r ? xcd : r) + i / 8u;
    }
    const uint32_t per_batch = p.tilesM * p.tilesN;
    const uint32_t b = pid / per_batch;
    const uint32_t pin = pid - b * per_batch;
    const uint32_t GM = 8, width = GM * p.tilesN;
    const uint32_t first_m = (pin / width) * GM;
    const uint32_t gsz = p.tilesM - first_m < GM ? p.tilesM - first_m : GM;
    const uint32_t tm_ = first_m + (pin % width) % gsz;
    const uint32_t tn_ = (pin % width) / gsz;
    const int64_t bm = (int64_t)tm_ * BM, bn = (int64_t)tn_ * BN;

    const double *A = p.A + (int64_t)b * p.strideA;
    const double *B = p.B + (int64_t)b * p.strideB;

    d4 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (d4){0.0, 0.0, 0.0, 0.0};

    const int nkt = (int)((p.K + BK - 1) / BK);
    // whole-tile operands take the unguarded loader (a uniform choice per k step)
    const bool fastA = p.vecA && bm + BM <= p.M, fastB = p.vecB && bn + BN <= p.N;
    const double *oa = tile_origin<KCA>(A, p.lda, bm), *ob = tile_origin<KCB>(B, p.ldb, bn);
    d2 ra[4], rb[4];
    auto fetch = [&](int64_t k0) {
        const bool kfull = k0 + BK <= p.K;
        if (fastA && kfull) load_tile_fast<KCA>(oa, p.lda, k0, ra);
        else load_tile<KCA>(A, p.lda, bm, k0, p.M, p.K, p.vecA, ra);
        if (fastB && kfull) load_tile_fast<KCB>(ob, p.ldb, k0, rb);
        else load_tile<KCB>(B, p.ldb, bn, k0, p.N, p.K, p.vecB, rb);
    };
    if (nkt > 0) {
        fetch((int64_t)(p.variant ? nkt - 1 : 0) * BK);
        store_tile<KCA>(lds, ra);
        store_tile<KCB>(lds + 2 * kTileDoubles, rb);
    }
    __syncthreads();
    int cur = 0;
    for (int it = 0; it < nkt; ++it) {
        const bool more = it + 1 < nkt;
        if (more) fetch((int64_t)(p.variant ? nkt - 2 - it : it + 1) * BK);
        const double *As = lds + cur * kTileDoubles + wm * 64 + (lane & 15);
        const double *Bs = lds + (2 + cur) * kTileDoubles + wn * 64 + (lane & 15);
        double a[4], bb[4];
#pragma unroll
        for (int kk = 0; kk < BK / 4; ++kk) {
            const int krow = (kk * 4 + (lane >> 4)) * LDS_S;
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[krow + i * 16]; bb[i] = Bs[krow + i * 16]; }
            if (kk == BK / 4 - 1) {
                // The next tile goes to the other LDS buffer in the shadow of the last 16 MFMAs
                // of this one (its fragments are already requested: LDS completes in order), so
                // a wave's MFMA stream has no gap before the barrier.
                __builtin_amdgcn_sched_barrier(0);
                if (more) {
                    store_tile<KCA>(lds + (cur ^ 1) * kTileDoubles, ra);
                    store_tile<KCB>(lds + (2 + (cur ^ 1)) * kTileDoubles, rb);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[i], bb[j], acc[i][j], 0, 0, 0);
        }
        __syncthreads();
        cur ^= 1;
    }

    // ---- epilogue: alpha, bias, round, decide, store, bit-planes -------------------------
    const int g = lane >> 4, c16 = lane & 15;
    const int64_t row0 = bm + wm * 64, col0 = bn + wn * 64;
    const uint64_t colword = (uint64_t)col0 >> 6;
    const bool word_exists = colword < p.wpr;
    float *C32 = p.C32 + (int64_t)b * p.strideC;
    double *C64 = p.C64 ? p.C64 + (int64_t)b * p.M * p.N : nullptr;
    double bias_v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int64_t col = col0 + j * 16 + c16;
        bias_v[j] = (p.bias && col < p.N) ? p.bias[col] : 0.0;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int64_t row = row0 + i * 16 + 4 * r + g;
            uint64_t lgw = 0, drw = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t col = col0 + j * 16 + c16;
                const bool in = row < p.M && col < p.N;
                double c = p.alpha * acc[i][j][r];
                if (p.bias) c = c + bias_v[j];
                const FastDecision f = decide_fast(c);
                uint32_t yb = __float_as_uint(f.y);
                bool logged = f.D < p.thr, up = f.grow != f.neg;
                if (__builtin_expect(__ballot(f.slow) != 0, 0)) {     // NaN, Inf, zero, tiny or huge values
                    if (f.slow) {
                        const Decision d = decide((uint64_t)__double_as_longlong(c));
                        yb = d.ybits; logged = d.D < p.thr; up = d.dir != 0;
                    }
                }
                if (in) {
                    C32[row * p.ldc + col] = __uint_as_float(yb);
                    if (C64) C64[row * p.N + col] = c;
                }
                const uint64_t lg = __ballot(in && logged);
                const uint64_t dr = __ballot(up) & lg;
                lgw |= ((lg >> (16 * g)) & 0xFFFFull) << (16 * j);
                drw |= ((dr >> (16 * g)) & 0xFFFFull) << (16 * j);
            }
            if (c16 == 0 && row < p.M && word_exists) {
                const uint64_t w = ((uint64_t)b * (uint64_t)p.M + (uint64_t)row) * p.wpr + colword;
                p.pl_logged[w] = lgw;
                p.pl_dir[w] = drw;
            }
        }
    }
}

}  // namespace

hipError_t launch_gemm_round_planes(const GemmArgs &g, const Planes &pl, hipStream_t s)
{
    GemmParams p;
    p.A = g.A; p.B = g.B; p.bias = g.bias; p.C32 = g.C32; p.C64 = g.C64;
    p.pl_logged = pl.logged; p.pl_dir = pl.dir;
    p.M = g.M; p.N = g.N; p.K = g.K; p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
    p.strideA = g.strideA; p.strideB = g.strideB; p.strideC = g.strideC;
    p.alpha = g.alpha; p.thr = g.thr; p.wpr = pl.wpr; p.variant = g.variant;
    p.tilesM = (uint32_t)((g.M + BM - 1) / BM);
    p.tilesN = (uint32_t)((g.N + BN - 1) / BN);
    const uint64_t total = (uint64_t)p.tilesM * p.tilesN * (uint64_t)g.batch;
    if (total == 0) return hipSuccess;
    if (total > 0x7FFFFFFFull) return hipErrorInvalidValue;
    p.total_tiles = (uint32_t)total;
    p.vecA = ((uintptr_t)g.A % 16 == 0) && (g.lda % 2 == 0) && (g.strideA % 2 == 0);
    p.vecB = ((uintptr_t)g.B % 16 == 0) && (g.ldb % 2 == 0) && (g.strideB % 2 == 0);
    const bool kca = !g.transA, kcb = g.transB != 0;
    const dim3 grid(p.total_tiles), block(256);
    if (kca && kcb) gemm_round_planes_kernel<true, true><<<grid, block, 0, s>>>(p);
    else if (kca && !kcb) gemm_round_planes_kernel<true, false><<<grid, block, 0, s>>>(p);
    else if (!kca && kcb) gemm_round_planes_kernel<false, true><<<grid, block, 0, s>>>(p);
    else gemm_round_planes_kernel<false, false><<<grid, block, 0, s>>>(p);
    return hipGetLastError();
}

}  // namespace vt
