// vt_gemm_tile.h -- FP64 MFMA GEMM with the trainer hook fused into its epilogue (gfx950).
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
// This header holds the kernel template; each workgroup tile shape is instantiated in a
// translation unit of its own (vt_gemm_shape_*.hip) so that they compile side by side.
#pragma once
#include "vt_device.h"
#include "vt_kernels.h"

#include <type_traits>

namespace vt {

// one entry point per workgroup tile shape (defined in vt_gemm_shape_*.hip)
struct GemmParams;
hipError_t launch_gemm_128x128(const GemmParams &p, int am, bool kcb, hipStream_t s);
hipError_t launch_gemm_64x64(const GemmParams &p, int am, bool kcb, hipStream_t s);

constexpr int BK = 16;

struct GemmParams {
    ConvGeom conv;
    const double *A, *B, *bias;
    float *C32;
    double *C64;                                // optional dense FP64 copy (fused path only)
    double *partial;                            // split-K slabs [split][batch][M][N]
    uint64_t *pl_logged, *pl_dir;
    int64_t M, N, K, lda, ldb, ldc, strideA, strideB, strideC, batch;
    int64_t strideA2, strideB2;                 // operand offsets between groups of batch_inner matrices
    uint32_t batch_inner;                       // matrix b uses group b / batch_inner, member b % batch_inner
    double alpha;
    uint32_t thr, wpr, tilesM, tilesN, tiles_per_split, total_blocks;
    uint32_t m_tiles_per_split, m_per_batch, m_width, m_batch_inner;   // divmod_magic multipliers of the tile mapping's divisors
    int variant, vecA, vecB, splits, kt_per_split, raw;
    uint32_t *zero_a, *zero_b;                  // words cleared by the kernel for the log compaction that follows
    uint32_t zero_a_words, zero_b_words;
    // Tail tiles: the tiles from number tail_first on are multiplied by 2^tail_shift workgroups each, every one a
    // slice of tail_kt k steps whose raw accumulators go to tail_partial (tile-sized slabs); gemm_tail_fixup_kernel
    // adds the slices in a fixed order and runs the epilogue.  Workgroup tail_first + (j << tail_shift) + s of the
    // launch is slice s of tail tile j.  tail_first = tiles_total: no tail.
    uint32_t tiles_total;                       // tiles x split-K slices: what the tile mapping counts
    uint32_t tail_first, tail_shift, tail_kt;
    double *tail_partial;
};

constexpr int kGroupMax = 4;
struct GemmGroup {
    GemmParams p[kGroupMax];
    uint32_t first[kGroupMax + 1];
};
hipError_t launch_gemm_grouped_128x128(const GemmGroup &gp, int am, bool kcb, hipStream_t s);
hipError_t launch_gemm_grouped_64x64(const GemmGroup &gp, int am, bool kcb, hipStream_t s);

namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));

// LDS row pitch = tile width + 18 doubles (128 x 128 tile) or + 14 (64 x 64 tile).  A k-contiguous operand is transposed on its way into
// LDS: the 32 lanes of a write pass hold 8 k rows x 4 columns, and with a pitch of 18 mod 32
// doubles those land on 32 different bank pairs (a pitch of 16 mod 32 put all 8 k rows on one
// pair: 8-way conflicts that kept the LDS pipe busy for about as long as the MFMAs).  Fragment
// reads (2 k rows x 16 columns per pass) then overlap in 2 of 32 bank pairs only.
// A pad of 14 has both properties as well (14 = 18 - 4: the same store pattern, reads overlapping
// in bank pairs 14 and 15); the 64x64 tile takes it, which brings its two stages under 40 KB so
// that four workgroups share a CU's LDS instead of three.
constexpr int kPad = 18, kPadSmall = 14;


// Two neighbouring taps of one row.  An element in the padding, outside the matrix or (input
// gradient) between the stride's positions is loaded from a pair of zeros instead: the choice is
// made on the address, so nothing has to wait for the loaded value before it goes to LDS two
// steps later, and the loop body stays free of branches.
static __device__ __attribute__((aligned(16))) double kZeroPair[2] = {0.0, 0.0};     // never written (not const: a global-memory address keeps the loads off the LDS counter)

template <bool VEC, bool UP = false>
__device__ __forceinline__ d2 conv_gather(const double *__restrict__ X, const ConvGeom &c, const RowPos &r,
                                          const TapPos &t0, const TapPos &t1)
{
    // UP (input gradient): the row's and the tap's stride remainders must agree as well
    const bool ok0 = (uint32_t)(r.h0 + t0.hh) < (uint32_t)c.H && (uint32_t)(r.w0 + t0.ww) < (uint32_t)c.W &&
                     (!UP || r.rem == t0.rem);
    const double *p0 = X + (r.base + t0.off);
    if (VEC) return *(const d2 *)(ok0 ? p0 : kZeroPair);
    const bool ok1 = (uint32_t)(r.h0 + t1.hh) < (uint32_t)c.H && (uint32_t)(r.w0 + t1.ww) < (uint32_t)c.W &&
                     (!UP || r.rem == t1.rem);
    const double *p1 = X + (r.base + t1.off);
    d2 v;
    v.x = *(ok0 ? p0 : kZeroPair);
    v.y = *(ok1 ? p1 : kZeroPair);
    return v;
}

// Global -> registers for one R x 16 operand tile (R = 64 or 128 rows/columns of the output).
// KC = the operand is contiguous along k (element (mn, k) at base[mn * ld + k]); otherwise
// contiguous along m/n (base[k * ld + mn]).  Each thread moves R / 32 pairs of doubles.
// Out-of-range elements read as 0, so partial tiles add exact zeros.
template <bool KC, int R>
__device__ __forceinline__ void load_tile(const double *__restrict__ base, int64_t ld, int64_t mn0, int64_t k0,
                                          int64_t MN, int64_t K, int vec, d2 (&regs)[R / 32])
{
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < R / 32; ++j) {
        int64_t mn, k;
        if (KC) { mn = mn0 + (t >> 3) + 32 * j; k = k0 + (t & 7) * 2; }
        else    { k = k0 + t / (R / 2) + (512 / R) * j; mn = mn0 + (t % (R / 2)) * 2; }
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

// Same tile when it lies wholly inside the operand and 16-byte loads are legal: straight vector
// loads, no guards.  Addresses are a workgroup-uniform base (scalar registers, advanced per k
// step) plus a per-thread 32-bit byte offset that never changes, so the loop spends no vector
// instructions -- and no load-destination registers -- on address arithmetic.
template <bool KC, int R>
__device__ __forceinline__ void tile_offsets(int64_t ld, uint32_t (&off)[R / 32])
{
    const int t = threadIdx.x;
#pragma unroll
    for (int j = 0; j < R / 32; ++j)
        off[j] = KC ? (uint32_t)((((t >> 3) + 32 * j) * ld + (t & 7) * 2) * 8)
                    : (uint32_t)(((t / (R / 2) + (512 / R) * j) * ld + (t % (R / 2)) * 2) * 8);
}

template <bool KC, int R>
__device__ __forceinline__ void load_tile_fast(const char *__restrict__ base, int64_t ld, int64_t k0,
                                               uint32_t (&off)[R / 32], d2 (&regs)[R / 32])
{
    const char *p = base + (KC ? k0 : k0 * ld) * 8;      // uniform
#pragma unroll
    for (int j = 0; j < R / 32; ++j) {
        // the offset is made opaque here so that its zero-extension stays next to the load: the load
        // then takes the scalar base and the 32-bit lane offset as they are, with no vector add
        asm volatile("" : "+v"(off[j]));
        regs[j] = *(const d2 *)(p + off[j]);
    }
}

template <bool KC, int R, int PAD>
__device__ __forceinline__ void store_tile(double *__restrict__ S, const d2 (&regs)[R / 32])
{
    const int t = threadIdx.x;
    constexpr int pitch = R + PAD;
#pragma unroll
    for (int j = 0; j < R / 32; ++j) {
        if (KC) {
            const int mn = (t >> 3) + 32 * j, k = (t & 7) * 2;
            S[k * pitch + mn] = regs[j].x;
            S[(k + 1) * pitch + mn] = regs[j].y;
        } else {
            const int k = t / (R / 2) + (512 / R) * j, mn = (t % (R / 2)) * 2;
            *(d2 *)&S[k * pitch + mn] = regs[j];
        }
    }
}

// Bits [16 q, 16 q + 16) of two wave-uniform 64-bit masks, side by side: a's in the low half.
__device__ __forceinline__ uint32_t pack16(uint64_t a, uint64_t b, int q)
{
    const uint32_t x = (uint32_t)(a >> (32 * (q >> 1))), y = (uint32_t)(b >> (32 * (q >> 1)));
    return (q & 1) ? (x >> 16) | (y & 0xFFFF0000u) : (x & 0xFFFFu) | (y << 16);
}

// v with lane `ln` (a compile-time constant) replaced by the wave-uniform value s.
__device__ __forceinline__ int write_lane(uint32_t s, int ln, int v)
{
    asm("v_writelane_b32 %0, %1, %2" : "+v"(v) : "s"(s), "n"(ln));
    return v;
}

// Work item id (a workgroup id, or a position in a persistent workgroup's list) -> (split, batch
// element, tile origin, operand bases).  Consecutive ids land on different XCDs (8 of them, each with
// its own L2), so ids are first regrouped per XCD, then walked in bands of 8 row tiles so that
// neighbours in time share A and B panels in that L2.  All wave-uniform: the divisors are run-time
// values, and multiply-high by reciprocals from the host keeps these splits on the scalar unit (the
// compiler's own division sequence runs on the vector unit).
template <int BM, int BN>
__device__ __forceinline__ void tile_of(const GemmParams &p, uint32_t id, uint32_t &split, uint32_t &b, int64_t &bm,
                                        int64_t &bn, const double *&A, const double *&B)
{
    uint32_t pid;
    {
        const uint32_t q = p.tiles_total / 8u, r = p.tiles_total % 8u, xcd = id % 8u;
        pid = xcd * q + (xcd < r ? xcd : r) + id / 8u;
    }
    uint32_t pin, band, inband, b_out, b_in;
    divmod_magic(pid, p.tiles_per_split, p.m_tiles_per_split, split, pid);
    const uint32_t per_batch = p.tilesM * p.tilesN;
    divmod_magic(pid, per_batch, p.m_per_batch, b, pin);
    const uint32_t GM = 8, width = GM * p.tilesN;
    divmod_magic(pin, width, p.m_width, band, inband);
    const uint32_t first_m = band * GM;
    const uint32_t gsz = p.tilesM - first_m < GM ? p.tilesM - first_m : GM;
    uint32_t tm_, tn_;
    if (gsz == GM) { tm_ = first_m + (inband & (GM - 1)); tn_ = inband / GM; }
    else { tm_ = first_m + inband % gsz; tn_ = inband / gsz; }       // the last, shorter band
    bm = (int64_t)tm_ * BM;
    bn = (int64_t)tn_ * BN;
    divmod_magic(b, p.batch_inner, p.m_batch_inner, b_out, b_in);
    A = p.A + (int64_t)b_out * p.strideA2 + (int64_t)b_in * p.strideA;
    B = p.B + (int64_t)b_out * p.strideB2 + (int64_t)b_in * p.strideB;
}

// The fused trainer hook on one wave's accumulators (16 TM rows x 64 columns at (row0, col0) of batch
// element b): alpha, bias, round to FP32, decide, store C32 (and the FP64 copy), decision bits to the
// two bit-planes.
template <int TM, int BM, int BN>
__device__ __forceinline__ void tile_epilogue(const GemmParams &p, const d4 (&acc)[TM][4], uint32_t b, int64_t bm, int64_t bn,
                                              int64_t row0, int64_t col0, int lane)
{
    const int g = lane >> 4, c16 = lane & 15;
    // ---- epilogue: alpha, bias, round, decide, store, bit-planes -------------------------
    const uint64_t colword = (uint64_t)col0 >> 6;
    // Whole tile inside the matrix (and pitches that fit 32-bit lane offsets): no guards, every
    // address is a wave-uniform base plus a lane offset that never changes, the four ballots of
    // a row group are transposed into plane words with scalar pack operations, and the rare
    // values that need the integer rounding path are handled once per group of four.
    if (bm + BM <= p.M && bn + BN <= p.N && p.ldc < (1 << 26) && p.N < (1 << 25)) {
        // PLAIN: alpha = 1 and no bias (every convolution): the product and the sum would return the
        // accumulator bit for bit, and each vector instruction here is paid in MFMA time
        auto full = [&](auto has64_tag, auto plain_tag) {
            constexpr bool HAS64 = decltype(has64_tag)::value, PLAIN = decltype(plain_tag)::value;
            const uint32_t win0 = thr_window_base(p.thr), win1 = thr_window_size(p.thr);
            const uint32_t nwin0 = 0u - win0, win1s = win1 << 3;
            char *c32_row = (char *)(p.C32 + (int64_t)b * p.strideC + row0 * p.ldc + col0);      // uniform, row 4 r of block i
            char *c64_row = HAS64 ? (char *)(p.C64 + ((int64_t)b * p.M + row0) * p.N + col0) : nullptr;
            const uint32_t step32 = (uint32_t)p.ldc * 16u, step64 = (uint32_t)p.N * 32u;         // four rows further
            const uint32_t off32 = ((uint32_t)g * (uint32_t)p.ldc + (uint32_t)c16) * 4u;
            const uint32_t off64 = ((uint32_t)g * (uint32_t)p.N + (uint32_t)c16) * 8u;
            char *wl_blk = (char *)(p.pl_logged + ((uint64_t)b * (uint64_t)p.M + (uint64_t)row0) * p.wpr + colword);
            char *wd_blk = (char *)(p.pl_dir + ((uint64_t)b * (uint64_t)p.M + (uint64_t)row0) * p.wpr + colword);
            const uint32_t offw = (uint32_t)(lane & 15) * p.wpr * 8u;                            // lane = row of the block
            double bias_f[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) bias_f[j] = p.bias ? p.bias[col0 + j * 16 + c16] : -0.0;   // x + (-0) = x
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                int wl_lo = 0, wl_hi = 0, wd_lo = 0, wd_hi = 0;       // lane q: plane words of row q of this block
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    double c[4];
                    uint32_t yb[4];
                    uint64_t lg[4], dr[4], slow[4], any_slow = 0;
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        c[j] = PLAIN ? acc[i][j][r] : p.alpha * acc[i][j][r] + bias_f[j];
                        const FastLogged f = decide_fast_window(c[j], win0, win1);
                        yb[j] = __float_as_uint(f.y);
                        // (the compare's lane mask itself: a ballot of the stored flag goes through a register)
                        lg[j] = __builtin_amdgcn_uicmp(window_key((uint32_t)__double_as_longlong(c[j]), nwin0), win1s, 36 /* unsigned < */);
                        dr[j] = __ballot(f.up) & lg[j];
                        // outside the FP32-normal range (exponent field below 897 or from 1151 up, NaN):
                        // two compares on |c| whose lane masks are the result
                        const double ac = __builtin_fabs(c[j]);
                        slow[j] = __builtin_amdgcn_fcmp(ac, 0x1p-126, 12 /* < or unordered */) |
                                  __builtin_amdgcn_fcmp(ac, 0x1p128, 11 /* >= or unordered */);
                        any_slow |= slow[j];
                    }
                    if (__builtin_expect(any_slow != 0, 0)) {          // NaN, Inf, zero, tiny or huge values
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const Decision d = decide((uint64_t)__double_as_longlong(c[j]));
                            const bool sl = (slow[j] >> lane) & 1;
                            if (sl) yb[j] = d.ybits;
                            const uint64_t lgs = __ballot(d.D < p.thr), drs = __ballot(d.dir != 0) & lgs;
                            lg[j] = (lg[j] & ~slow[j]) | (lgs & slow[j]);
                            dr[j] = (dr[j] & ~slow[j]) | (drs & slow[j]);
                        }
                    }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        *(float *)(c32_row + off32 + j * 64) = __uint_as_float(yb[j]);
                        if (HAS64) *(double *)(c64_row + off64 + j * 128) = c[j];
                    }
                    c32_row += step32;
                    if (HAS64) c64_row += step64;
                    // 16-bit group q of the four ballots -> plane word of row 4 r + q (scalar packs),
                    // parked in lane 4 r + q until the block's sixteen rows are complete
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int ln = 4 * r + q;
                        wl_lo = write_lane(pack16(lg[0], lg[1], q), ln, wl_lo);
                        wl_hi = write_lane(pack16(lg[2], lg[3], q), ln, wl_hi);
                        wd_lo = write_lane(pack16(dr[0], dr[1], q), ln, wd_lo);
                        wd_hi = write_lane(pack16(dr[2], dr[3], q), ln, wd_hi);
                    }
                }
                if (lane < 16) {
                    *(uint64_t *)(wl_blk + offw) = ((uint64_t)(uint32_t)wl_hi << 32) | (uint32_t)wl_lo;
                    *(uint64_t *)(wd_blk + offw) = ((uint64_t)(uint32_t)wd_hi << 32) | (uint32_t)wd_lo;
                }
                wl_blk += (uint64_t)p.wpr * 128u;
                wd_blk += (uint64_t)p.wpr * 128u;
            }
        };
        const bool plain = p.alpha == 1.0 && !p.bias;
        if (p.C64) { if (plain) full(std::true_type{}, std::true_type{}); else full(std::true_type{}, std::false_type{}); }
        else { if (plain) full(std::false_type{}, std::true_type{}); else full(std::false_type{}, std::false_type{}); }
        return;
    }
    // edge tiles: every access guarded
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
    for (int i = 0; i < TM; ++i) {
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

// AM, the A operand: 0 = stored transposed (contiguous along m), 1 = row-major (contiguous along
// k), 2 = implicit im2col of an image, rows x taps (convolution forward), 3 = its transpose,
// taps x rows (convolution weight gradient), 4 = the input-gradient view of the output gradient,
// input positions x (filter position, output channel).  KCB: B is stored transposed (contiguous along k).
// `bid` of `nblk`: the workgroup's number among those of this problem (the launch may hold several problems)
template <int AM, bool KCB, int WM, int TM>
__device__ __forceinline__ void gemm_tile_body(const GemmParams &p, const uint32_t bid, const uint32_t nblk)
{
    constexpr bool KCA = AM == 1 || AM == 2 || AM == 4;
    constexpr bool GA = AM >= 2;
    constexpr int WN = 4 / WM;
    constexpr int BM = WM * 16 * TM, BN = WN * 64;
    constexpr int PAD = TM == 1 ? kPadSmall : kPad;
    constexpr int PA = BM + PAD, PB = BN + PAD;            // LDS pitches
    constexpr int SA = BK * PA, SB = BK * PB;              // doubles per stage
    __shared__ double lds[2 * SA + 2 * SB];                // A0 A1 B0 B1
    double *const ldsA = lds, *const ldsB = lds + 2 * SA;
    const int t = threadIdx.x, lane = t & 63;
    const int wv = __builtin_amdgcn_readfirstlane(t >> 6);      // wave-uniform: keeps tile addresses in scalar registers
    const int wm = wv / WN, wn = wv % WN;

    // what the single-launch log compaction after this kernel needs zeroed: its status words and the
    // direction words of the log (a few words per workgroup)
    for (uint32_t i = bid * 256u + t; i < p.zero_a_words; i += nblk * 256u) p.zero_a[i] = 0u;
    for (uint32_t i = bid * 256u + t; i < p.zero_b_words; i += nblk * 256u) p.zero_b[i] = 0u;

    // a tail tile is shared by several workgroups, each a slice of its k range (uniform over the workgroup)
    const bool tail = bid >= p.tail_first;
    uint32_t tile_id = bid, tail_slice = 0;
    if (tail) {
        const uint32_t j = bid - p.tail_first;
        tile_id = p.tail_first + (j >> p.tail_shift);
        tail_slice = j & ((1u << p.tail_shift) - 1u);
    }
    uint32_t split, b;
    int64_t bm, bn;
    const double *A, *B;
    tile_of<BM, BN>(p, tile_id, split, b, bm, bn, A, B);

    d4 acc[TM][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = (d4){0.0, 0.0, 0.0, 0.0};

    // this workgroup's k tiles: [kt0, kt1)
    const int nkt_all = (int)((p.K + BK - 1) / BK);
    const int kt_len = tail ? (int)p.tail_kt : p.kt_per_split;
    const int kt0 = (int)(tail ? tail_slice : split) * kt_len;
    const int kt1 = kt0 + kt_len < nkt_all ? kt0 + kt_len : nkt_all;
    const int nkt = kt1 > kt0 ? kt1 - kt0 : 0;
    // whole-tile operands take the unguarded loader (a uniform choice per k step)
    // (the per-thread offsets of the unguarded loader are 32-bit: pitches up to 2^31 / 8 / 128)
    const bool fastA = GA ? p.conv.vec != 0 : p.vecA && bm + BM <= p.M && p.lda < (1 << 21);
    const bool fastB = p.vecB && bn + BN <= p.N && p.ldb < (1 << 21);
    const char *baseA = (const char *)(A + (KCA ? bm * p.lda : bm));
    const char *baseB = (const char *)(B + (KCB ? bn * p.ldb : bn));
    uint32_t offA[BM / 32], offB[BN / 32];
    tile_offsets<KCA, BM>(p.lda, offA);
    tile_offsets<KCB, BN>(p.ldb, offB);
    // Two register sets: tile it+2 is in flight from memory while tile it+1 (fetched one step
    // earlier) goes to LDS and tile it is multiplied, so a fetch has two full steps to land.
    // The loop exists twice: with unguarded loads only (every tile of this workgroup lies inside
    // the operands; straight-line code, so the load counter waits are exact and the newest
    // fetch stays in flight across the LDS stores), and with the guarded loader for edges.
    d2 ra0[BM / 32], rb0[BN / 32], ra1[BM / 32], rb1[BN / 32];
    // Implicit im2col: the part of the address that belongs to this thread for the whole loop --
    // its rows of the image matrix (forward) or its pair of taps (weight gradient).
    RowPos rowp[AM == 2 || AM == 4 ? BM / 32 : 1];
    TapPos tap0{0, 0, 0, 0}, tap1{0, 0, 0, 0};
    if constexpr (AM == 2) {
#pragma unroll
        for (int j = 0; j < BM / 32; ++j) rowp[j] = conv_row(p.conv, (uint32_t)bm + (t >> 3) + 32 * j);
    }
    if constexpr (AM == 4) {
#pragma unroll
        for (int j = 0; j < BM / 32; ++j) rowp[j] = dgrad_row(p.conv, (uint32_t)bm + (t >> 3) + 32 * j);
    }
    // (weight gradient: the rows run along k; each thread walks its BM / 32 rows a k step at a time,
    // from the first tile it fetches, in the variant's direction)
    // (the large tile has no registers left for the walk: there a k step's row t / 64 + 4 j is the same for a
    // whole wave and is split in scalar registers, 6 % faster than splitting it per thread; the same
    // per half-wave for the small tile measured 10 % slower than the walk)
    constexpr bool WALK = AM == 3 && BM == 64;
    RowIter rit[WALK ? BM / 32 : 1];
    int32_t row_an = 0, row_ah = 0, row_aw = 0;
    if constexpr (AM == 3) {
        const uint32_t kc = (uint32_t)bm + (t % (BM / 2)) * 2;
        tap0 = conv_tap(p.conv, kc);
        tap1 = conv_tap(p.conv, kc + 1);
    }
    if constexpr (WALK) {
        static_assert(BK == kRowStep, "the row walk advances one k step at a time");
        const uint32_t kfirst = (uint32_t)(p.variant ? kt1 - 1 : kt0) * BK;
#pragma unroll
        for (int j = 0; j < BM / 32; ++j) rit[j] = row_iter(p.conv, kfirst + t / (BM / 2) + (512 / BM) * j);
        row_step_digits(p.conv, p.variant != 0, row_an, row_ah, row_aw);
    }
    // UNI: the channel count is a multiple of 16, so the 16 taps of a k step are 16 channels of one
    // filter position: (kh, kw) and the tap's offset are the same for the whole wave and are found
    // with scalar integer operations; the lane's channel pair is already part of its rows' offsets.
    auto gather_tile = [&](auto vec_tag, auto uni_tag, int64_t k0, d2 (&ra)[BM / 32]) {
        constexpr bool VEC = decltype(vec_tag)::value, UNI = decltype(uni_tag)::value;
        if constexpr (UNI && (AM == 2 || AM == 4)) {
            const TapPos t0 = AM == 2 ? conv_tap<true>(p.conv, (uint32_t)k0) : dgrad_tap<true>(p.conv, (uint32_t)k0);
#pragma unroll
            for (int j = 0; j < BM / 32; ++j) ra[j] = conv_gather<true, AM == 4>(p.A, p.conv, rowp[j], t0, t0);
        } else if constexpr (AM == 2) {
            const uint32_t kc = (uint32_t)k0 + (t & 7) * 2;
            const TapPos t0 = conv_tap(p.conv, kc);
            const TapPos t1 = VEC ? t0 : conv_tap(p.conv, kc + 1);
#pragma unroll
            for (int j = 0; j < BM / 32; ++j) ra[j] = conv_gather<VEC>(p.A, p.conv, rowp[j], t0, t1);
        } else if constexpr (AM == 3) {
#pragma unroll
            for (int j = 0; j < BM / 32; ++j) {
                if constexpr (WALK) {
                    // the tiles are fetched in order, one per call (a fetch repeated past the last
                    // tile moves on to rows nobody multiplies): k0 is implied
                    ra[j] = conv_gather<VEC>(p.A, p.conv, row_pos(p.conv, rit[j]), tap0, tap1);
                    row_advance(p.conv, rit[j], row_an, row_ah, row_aw);
                } else {
                    static_assert(BM == 128, "row t / (BM / 2) + (512 / BM) j is wave-uniform for the large tile only");
                    const RowPos r = conv_row<true>(p.conv, (uint32_t)k0 + (uint32_t)wv + 4u * j);
                    ra[j] = conv_gather<VEC>(p.A, p.conv, r, tap0, tap1);
                }
            }
        } else if constexpr (AM == 4) {
            const uint32_t kc = (uint32_t)k0 + (t & 7) * 2;
            const TapPos t0 = dgrad_tap(p.conv, kc);
            const TapPos t1 = VEC ? t0 : dgrad_tap(p.conv, kc + 1);
#pragma unroll
            for (int j = 0; j < BM / 32; ++j) ra[j] = conv_gather<VEC, true>(p.A, p.conv, rowp[j], t0, t1);
        }
    };
    auto main_loop = [&](auto fast_tag, auto uni_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        auto fetch = [&](int it, d2 (&ra)[BM / 32], d2 (&rb)[BN / 32]) {   // `it`-th step in this variant's order
            const int64_t k0 = (int64_t)(p.variant ? kt1 - 1 - it : kt0 + it) * BK;
            if constexpr (GA) {
                if constexpr (FAST) gather_tile(std::true_type{}, uni_tag, k0, ra);
                else if (p.conv.vec) gather_tile(std::true_type{}, std::false_type{}, k0, ra);
                else gather_tile(std::false_type{}, std::false_type{}, k0, ra);
            } else if constexpr (FAST) {
                load_tile_fast<KCA, BM>(baseA, p.lda, k0, offA, ra);
            } else {
                load_tile<KCA, BM>(A, p.lda, bm, k0, p.M, p.K, p.vecA, ra);
            }
            if constexpr (FAST) load_tile_fast<KCB, BN>(baseB, p.ldb, k0, offB, rb);
            else load_tile<KCB, BN>(B, p.ldb, bn, k0, p.N, p.K, p.vecB, rb);
        };
        // multiply the tile in LDS stage `cur`; with `more`, move the next tile from (sa, sb) to the other
        // stage in the shadow of the last MFMA group
        auto compute = [&](int cur, bool more, d2 (&sa)[BM / 32], d2 (&sb)[BN / 32]) {
            const double *As = ldsA + cur * SA + wm * (16 * TM) + (lane & 15);
            const double *Bs = ldsB + cur * SB + wn * 64 + (lane & 15);
            // The narrow tiles have registers to spare: the fragments of group kk + 1 are requested
            // before the MFMAs of group kk are issued, so an LDS round trip hides behind a whole
            // group instead of behind its last instruction.  (The large tile has none to spare; there
            // the compiler interleaves the reads as fragment registers fall free.)
            constexpr bool PIPE = TM <= 2;
            double a[PIPE ? 2 : 1][TM], bb[PIPE ? 2 : 1][4];
            auto frags = [&](int kk, double (&fa)[TM], double (&fb)[4]) {
                const int krow = kk * 4 + (lane >> 4);
#pragma unroll
                for (int i = 0; i < TM; ++i) fa[i] = As[krow * PA + i * 16];
#pragma unroll
                for (int j = 0; j < 4; ++j) fb[j] = Bs[krow * PB + j * 16];
            };
            if (PIPE) frags(0, a[0], bb[0]);
#pragma unroll
            for (int kk = 0; kk < BK / 4; ++kk) {
                const int cb = PIPE ? (kk & 1) : 0;
                if (!PIPE) frags(kk, a[0], bb[0]);
                else if (kk + 1 < BK / 4) {
                    frags(kk + 1, a[cb ^ 1], bb[cb ^ 1]);
                    __builtin_amdgcn_sched_barrier(0);         // keep the reads ahead of this group's MFMAs
                }
                if (kk == BK / 4 - 1) {
                    // (the last group's fragments are already requested: LDS completes in order,
                    // so the wave's MFMA stream has no gap before the barrier)
                    __builtin_amdgcn_sched_barrier(0);
                    if (more) {
                        store_tile<KCA, BM, PAD>(ldsA + (cur ^ 1) * SA, sa);
                        store_tile<KCB, BN, PAD>(ldsB + (cur ^ 1) * SB, sb);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(a[cb][i], bb[cb][j], acc[i][j], 0, 0, 0);
            }
            __syncthreads();
        };
        // one k step: start the fetch of tile it+2 into (la, lb); multiply tile it; tile it+1 goes from
        // (sa, sb) to LDS
        auto step = [&](int it, int cur, d2 (&la)[BM / 32], d2 (&lb)[BN / 32], d2 (&sa)[BM / 32], d2 (&sb)[BN / 32]) {
            // In the unguarded loop the fetch and the LDS store are unconditional (past the end
            // they repeat the last tile and fill a stage nobody reads): with no branch around
            // them the compiler's load-counter waits are exact.
            if (FAST) fetch(it + 2 < nkt ? it + 2 : nkt - 1, la, lb);
            else if (it + 2 < nkt) fetch(it + 2, la, lb);
            compute(cur, FAST || it + 1 < nkt, sa, sb);
        };
        if (nkt > 0) {
            fetch(0, ra0, rb0);
            store_tile<KCA, BM, PAD>(ldsA, ra0);
            store_tile<KCB, BN, PAD>(ldsB, rb0);
            if (nkt > 1) fetch(1, ra0, rb0);
        }
        __syncthreads();
        // (the odd last step stands after the loop: an exit from the middle of the body would reach
        // the loop's head with the first step's loads pending, and every wait in the body is placed
        // for the worst of the paths into it)
        int it = 0;
        for (; it + 1 < nkt; it += 2) {
            step(it, 0, ra1, rb1, ra0, rb0);                // tile it+1 sits in set 0, it+2 goes to set 1
            step(it + 1, 1, ra0, rb0, ra1, rb1);
        }
        if (it < nkt) step(it, 0, ra1, rb1, ra0, rb0);
    };
    const bool fast = fastA && fastB && (int64_t)kt1 * BK <= p.K;
    if ((AM == 2 || AM == 4) && fast && p.conv.uni) {
#pragma unroll
        for (int j = 0; j < BM / 32; ++j) rowp[j].base += (t & 7) * 2;
        main_loop(std::true_type{}, std::true_type{});
    } else if (fast) {
        main_loop(std::true_type{}, std::false_type{});
    } else {
        main_loop(std::false_type{}, std::false_type{});
    }

    const int g = lane >> 4, c16 = lane & 15;
    const int64_t row0 = bm + wm * (16 * TM), col0 = bn + wn * 64;

    if (tail) {
        // ---- a slice of a tail tile: raw accumulators to this workgroup's slab, rows and columns of the tile
        double *P = p.tail_partial + (uint64_t)(bid - p.tail_first) * (uint64_t)(BM * BN) + (wm * (16 * TM) + g) * BN + wn * 64 + c16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < 4; ++j) P[(i * 16 + 4 * r) * BN + j * 16] = acc[i][j][r];
        return;
    }
    if (p.splits > 1 || p.raw) {
        // ---- split-K (or a caller that rounds in a later pass): raw accumulators to this slice's slab; alpha, bias, rounding come later
        double *P = p.partial + ((int64_t)split * p.batch + (int64_t)b) * p.M * p.N;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int64_t row = row0 + i * 16 + 4 * r + g;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int64_t col = col0 + j * 16 + c16;
                    if (row < p.M && col < p.N) P[row * p.N + col] = acc[i][j][r];
                }
            }
        return;
    }

    tile_epilogue<TM, BM, BN>(p, acc, b, bm, bn, row0, col0, lane);
}

template <int AM, bool KCB, int WM, int TM>
__global__ __launch_bounds__(256, 2) void gemm_round_planes_kernel(const GemmParams p)
{
    gemm_tile_body<AM, KCB, WM, TM>(p, blockIdx.x, gridDim.x);
}

// Several problems of one tile shape and operand mode in one launch: workgroups first[g] .. first[g + 1] - 1
// belong to problem g (an empty problem has first[g] = first[g + 1]).  The stride phases of an input
// gradient are four small GEMMs of different depth; apart, each leaves most of the part idle.
template <int AM, bool KCB, int WM, int TM>
__global__ __launch_bounds__(256, 2) void gemm_grouped_kernel(const GemmGroup gp)
{
    uint32_t g = 0;
#pragma unroll
    for (int i = 1; i < kGroupMax; ++i)
        if (blockIdx.x >= gp.first[i]) g = i;
    gemm_tile_body<AM, KCB, WM, TM>(gp.p[g], blockIdx.x - gp.first[g], gp.first[g + 1] - gp.first[g]);
}

template <int WM, int TM>
hipError_t launch_shape_grouped(const GemmGroup &gp, int am, bool kcb, hipStream_t s)
{
    const dim3 grid(gp.first[kGroupMax]), block(256);
    if (am == 4 && !kcb) gemm_grouped_kernel<4, false, WM, TM><<<grid, block, 0, s>>>(gp);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// The tail tiles' slices added in ascending (variant 0) or descending slice order, then the fused epilogue: one
// workgroup per tail tile, every wave the rows and columns it would own in the GEMM kernel.
template <int WM, int TM>
__global__ __launch_bounds__(256) void gemm_tail_fixup_kernel(const GemmParams p)
{
    constexpr int WN = 4 / WM;
    constexpr int BM = WM * 16 * TM, BN = WN * 64;
    const int t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const int wm = wv / WN, wn = wv % WN, g = lane >> 4, c16 = lane & 15;
    uint32_t split, b;
    int64_t bm, bn;
    const double *A, *B;
    tile_of<BM, BN>(p, p.tail_first + blockIdx.x, split, b, bm, bn, A, B);
    const uint32_t S = 1u << p.tail_shift;
    d4 acc[TM][4];
    for (uint32_t q = 0; q < S; ++q) {
        const uint32_t sl = p.variant ? S - 1u - q : q;
        const double *P = p.tail_partial + ((uint64_t)blockIdx.x * S + sl) * (uint64_t)(BM * BN) + (wm * (16 * TM) + g) * BN + wn * 64 + c16;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const double v = P[(i * 16 + 4 * r) * BN + j * 16];
                    acc[i][j][r] = q == 0 ? v : acc[i][j][r] + v;
                }
    }
    tile_epilogue<TM, BM, BN>(p, acc, b, bm, bn, bm + wm * (16 * TM), bn + wn * 64, lane);
}

template <int WM, int TM>
hipError_t launch_shape(const GemmParams &p, int am, bool kcb, hipStream_t s)
{
    const dim3 grid(p.total_blocks), block(256);
    if (am == 2 && !kcb) gemm_round_planes_kernel<2, false, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 3 && !kcb) gemm_round_planes_kernel<3, false, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 4 && !kcb) gemm_round_planes_kernel<4, false, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 1 && kcb) gemm_round_planes_kernel<1, true, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 1 && !kcb) gemm_round_planes_kernel<1, false, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 0 && kcb) gemm_round_planes_kernel<0, true, WM, TM><<<grid, block, 0, s>>>(p);
    else if (am == 0 && !kcb) gemm_round_planes_kernel<0, false, WM, TM><<<grid, block, 0, s>>>(p);
    else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && p.tail_first < p.tiles_total) {
        gemm_tail_fixup_kernel<WM, TM><<<p.tiles_total - p.tail_first, 256, 0, s>>>(p);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace

}  // namespace vt
