// vt_device.h -- per-element device arithmetic of the round/log/replay path (gfx950).
//
// The definitions (decide, decide_slow, decide_k, directed_*) work on the binary64 bit pattern with
// integer instructions only.  The fast forms the kernels use for FP32-normal results (decide_fast,
// decide_fast_window) take the FP32 value from the hardware conversion v_cvt_f32_f64 instead, which
// equals rnd_32 only under round-to-nearest-even: they rely on the wave's MODE register holding the
// default FP64 rounding mode.  HIP launches every kernel in that mode and no kernel of this library
// changes it (no s_setreg, no directed-rounding intrinsics), which is what keeps the invariant; the
// conversion is restricted to 2^-126 <= |x| < 2^128 so that the denormal MODE bits cannot matter, and
// the distance and the direction always come from the dropped bits.  Both forms are held to each other
// and to the CPU oracle bit for bit by the host and GPU tests.
//
// For a finite x with |x| >= 2^-126 the FP32 result keeps the top 23 mantissa bits; the 29
// dropped bits r decide the rounding (Method, primitive rnd with b_r = 32):
//     r > 2^28, or r == 2^28 with an odd kept mantissa  ->  magnitude rounds up.
// The distance from x to the nearest FP32 midpoint, in FP64 steps, is D = |r - 2^28|; an output
// is logged iff D < thr (Algorithm "log" with tau = (0.5 - thr 2^-29) 2^-23, rewritten as a
// distance from the boundary instead of from the rounded value).  The direction bit is 1 iff
// the rounded value is greater than x (the paper's code 2).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vt {

constexpr uint32_t kHalf = 1u << 28;        // 2^28: half an FP32 ulp in FP64 steps
constexpr uint32_t kMask29 = (1u << 29) - 1;
constexpr uint32_t kF32Inf = 0x7F800000u;
constexpr uint32_t kF32QNaN = 0x7FC00000u;

struct Decision {
    uint32_t ybits;   // rnd_32(x) as a bit pattern
    uint32_t D;       // boundary distance in threshold units, in [0, 2^28]
    uint32_t dir;     // 1 iff rnd_32(x) > x (meaningful when x is not an FP32 value)
};

// Rare inputs: NaN, +-Inf, zero and every magnitude below 2^-126 (FP32 subnormal results,
// spacing fixed at 2^-149).  In that range the value is re-expressed on the 2^-178 grid
// (2^-29 of the FP32 spacing): q = floor(|x| / 2^-178), sticky = any finer bit set.
static __host__ __device__ __forceinline__ Decision decide_slow(uint64_t bits)
{
    const uint32_t sign = (uint32_t)(bits >> 63);
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    Decision o;
    if (mag > 0x7FF0000000000000ull) { o.ybits = kF32QNaN; o.D = kHalf; o.dir = 0; return o; }
    if (mag == 0x7FF0000000000000ull) { o.ybits = (sign << 31) | kF32Inf; o.D = kHalf; o.dir = 0; return o; }
    const uint32_t eb = (uint32_t)(mag >> 52);                       // biased exponent, < 897 here
    const uint64_t sig = eb ? ((mag & 0x000FFFFFFFFFFFFFull) | (1ull << 52)) : mag;
    const uint32_t sh = eb ? 897u - eb : 896u;                       // bits finer than 2^-178
    uint64_t q = 0;
    uint32_t sticky;
    if (sh > 63) { sticky = sig != 0; }
    else { q = sig >> sh; sticky = (sig & ((1ull << sh) - 1)) != 0; }
    const uint32_t r = (uint32_t)q & kMask29;
    uint32_t t = (uint32_t)(q >> 29);
    const uint32_t up = (r > kHalf) || (r == kHalf && (sticky || (t & 1u)));
    o.D = r >= kHalf ? r - kHalf : kHalf - r - sticky;
    t += up;                                                         // may become 2^-126, the smallest normal
    o.ybits = (sign << 31) | t;
    o.dir = up ^ sign;
    return o;
}

static __host__ __device__ __forceinline__ Decision decide(uint64_t bits)
{
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    const uint32_t ahi = hi & 0x7FFFFFFFu;
    // biased exponent in [897, 2046]: finite, |x| >= 2^-126
    if (__builtin_expect(ahi - (897u << 20) < ((2047u - 897u) << 20), 1)) {
        const uint32_t sign = hi >> 31;
        const uint32_t r = lo & kMask29;
        const uint32_t e = ahi - (896u << 20);                        // exponent re-biased for FP32
        Decision o;
        o.D = r > kHalf ? r - kHalf : kHalf - r;
        uint32_t t, up;
        if (__builtin_expect(e >= (255u << 20), 0)) {                 // |x| >= 2^128: overflows
            t = kF32Inf; up = 1;
        } else {
            t = (e << 3) | (lo >> 29);
            up = (r > kHalf) || (r == kHalf && (t & 1u));
            t += up;                                                  // a mantissa carry bumps the exponent; 0x7F800000 = Inf
        }
        o.ybits = (sign << 31) | t;
        o.dir = up ^ sign;
        return o;
    }
    return decide_slow(bits);
}

// Branch-free form of decide() for the streaming kernels, valid when `slow` comes back false,
// i.e. for finite x with 2^-126 <= |x| < 2^128.  There the FP32 result is a normal number (or
// overflows to infinity from the top binade), so the hardware conversion under the default
// round-to-nearest-even mode gives rnd_32(x) without touching denormal handling; the dropped
// bits still decide D and the direction: the magnitude grows iff r + (kept LSB) > 2^28.
// Lanes with slow == true must be redone with decide() (NaN, Inf, tiny, |x| >= 2^128); for +-0,
// which also comes back slow, y and D = 2^28 (never logged) are already right.
struct FastDecision {
    float y;
    uint32_t D;
    bool grow;      // magnitude rounded up
    bool neg;       // sign bit of x
    bool slow;
};

__device__ __forceinline__ FastDecision decide_fast(double x)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(x);
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    FastDecision o;
    o.slow = ((hi & 0x7FFFFFFFu) - (897u << 20)) >= ((1151u - 897u) << 20);
    const uint32_t r = lo & kMask29;
    o.D = __usad(r, kHalf, 0u);                     // |r - 2^28|
    o.grow = r + ((lo >> 29) & 1u) > kHalf;
    o.neg = (int32_t)hi < 0;
    o.y = (float)x;
    return o;
}

// The same decision with the threshold test folded into one subtraction and one unsigned compare,
// and the direction taken by value: D(x) < thr  <=>  (r - c0) <u c1 with c0 = 2^28 - thr + 1 and
// c1 = 2 thr - 1 (thr = 0: c1 = 0, never true), since |r - 2^28| < thr means r lies in
// [2^28 - thr + 1, 2^28 + thr - 1]; and rnd(x) > x is asked of the converted value itself (exact:
// every float is a double).  Four vector instructions fewer per output than decide_fast + compares,
// which is what the GEMM epilogue is made of.
struct FastLogged {
    float y;
    bool logged, up, slow;
};

static __host__ __device__ __forceinline__ uint32_t thr_window_base(uint32_t thr) { return kHalf - thr + 1u; }
static __host__ __device__ __forceinline__ uint32_t thr_window_size(uint32_t thr) { return thr ? 2u * thr - 1u : 0u; }
// The same test in one add-and-shift and one compare on the whole low word `lo` of the value:
// window_key(lo, 0 - base) < size << 3.  The shift by 3 drops the same top bits as the 29-bit mask,
// and dropped bits below the window wrap to 2^29 - base + r, which is >= size for every thr <= 2^28.
static __host__ __device__ __forceinline__ uint32_t window_key(uint32_t lo, uint32_t neg_base) { return (lo + neg_base) << 3; }

__device__ __forceinline__ FastLogged decide_fast_window(double x, uint32_t c0, uint32_t c1)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(x);
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    FastLogged o;
    o.slow = ((hi & 0x7FFFFFFFu) - (897u << 20)) >= ((1151u - 897u) << 20);
    o.logged = ((lo & kMask29) - c0) < c1;
    o.y = (float)x;
    o.up = (double)o.y > x;
    return o;
}

// Replay of one logged element (primitive "rev"): the FP32 neighbour of x on the logged side,
// i.e. x rounded toward +inf (dir = 1) or toward -inf (dir = 0).
static __host__ __device__ __forceinline__ uint32_t directed_slow(uint64_t bits, uint32_t dir)
{
    const uint32_t sign = (uint32_t)(bits >> 63);
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    if (mag > 0x7FF0000000000000ull) return kF32QNaN;
    if (mag == 0x7FF0000000000000ull) return (sign << 31) | kF32Inf;
    const uint32_t eb = (uint32_t)(mag >> 52);
    const uint64_t sig = eb ? ((mag & 0x000FFFFFFFFFFFFFull) | (1ull << 52)) : mag;
    const uint32_t sh = eb ? 897u - eb : 896u;
    uint64_t q = 0;
    uint32_t inexact;
    if (sh > 63) { inexact = sig != 0; }
    else { q = sig >> sh; inexact = (sig & ((1ull << sh) - 1)) != 0; }
    inexact |= ((uint32_t)q & kMask29) != 0;
    const uint32_t t = (uint32_t)(q >> 29) + (inexact & (dir ^ sign));
    return (sign << 31) | t;
}

static __host__ __device__ __forceinline__ uint32_t directed(uint64_t bits, uint32_t dir)
{
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    const uint32_t ahi = hi & 0x7FFFFFFFu;
    if (__builtin_expect(ahi - (897u << 20) < ((2047u - 897u) << 20), 1)) {
        const uint32_t sign = hi >> 31;
        const uint32_t away = dir ^ sign;                             // rounding grows the magnitude
        const uint32_t e = ahi - (896u << 20);
        uint32_t t;
        if (__builtin_expect(e >= (255u << 20), 0)) t = away ? kF32Inf : 0x7F7FFFFFu;   // |x| >= 2^128
        else t = ((e << 3) | (lo >> 29)) + (((lo & kMask29) != 0) & away);
        return (sign << 31) | t;
    }
    return directed_slow(bits, dir);
}

// ---- rounding amounts b_r < 32 -------------------------------------------------------------
// The target grid is the 32-bit floats whose last k = 32 - b_r mantissa bits are zero: spacing
// 2^k ulp32.  With T the FP32 pattern of |x| truncated (exponent and 23 mantissa bits) and r the
// 29 bits FP64 carries beyond it, the bits dropped by the coarser grid are R = (T mod 2^k) 2^29 + r
// (29 + k of them), the rounding boundary is R = 2^(28+k), and the kept pattern is T >> k.  The
// distance is reported in units of 2^k FP64 steps (2^-29 of the grid spacing), so thresholds
// keep their meaning relative to the spacing.  k = 0 gives decide() and directed().
static __host__ __device__ __forceinline__ Decision decide_k(uint64_t bits, uint32_t k)
{
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    const uint32_t sign = hi >> 31, ahi = hi & 0x7FFFFFFFu;
    const uint32_t maskk = (1u << k) - 1u;
    const uint64_t half = 1ull << (28 + k);
    Decision o;
    if (__builtin_expect(ahi - (897u << 20) < ((2047u - 897u) << 20), 1)) {      // finite, |x| >= 2^-126
        const uint32_t m23 = ((hi & 0xFFFFFu) << 3) | (lo >> 29);
        const uint64_t R = ((uint64_t)(m23 & maskk) << 29) | (lo & kMask29);
        o.D = (uint32_t)((R > half ? R - half : half - R) >> k);
        const uint32_t e = ahi - (896u << 20);
        uint32_t t, up;
        if (__builtin_expect(e >= (255u << 20), 0)) { t = kF32Inf; up = 1; }     // |x| >= 2^128: overflows
        else {
            const uint32_t P = ((e << 3) | (lo >> 29)) >> k;
            up = (R > half) || (R == half && (P & 1u));
            t = (P + up) << k;                                                   // carries reach 0x7F800000 = Inf
        }
        o.ybits = (sign << 31) | t;
        o.dir = up ^ sign;
        return o;
    }
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    if (mag > 0x7FF0000000000000ull) { o.ybits = kF32QNaN; o.D = kHalf; o.dir = 0; return o; }
    if (mag == 0x7FF0000000000000ull) { o.ybits = (sign << 31) | kF32Inf; o.D = kHalf; o.dir = 0; return o; }
    const uint32_t eb = (uint32_t)(mag >> 52);                       // below 2^-126: fixed spacing 2^(-149 + k)
    const uint64_t sig = eb ? ((mag & 0x000FFFFFFFFFFFFFull) | (1ull << 52)) : mag;
    const uint32_t sh = eb ? 897u - eb : 896u;
    uint64_t q = 0;
    uint32_t sticky;
    if (sh > 63) { sticky = sig != 0; }
    else { q = sig >> sh; sticky = (sig & ((1ull << sh) - 1)) != 0; }
    const uint32_t t0 = (uint32_t)(q >> 29);
    const uint64_t R = ((uint64_t)(t0 & maskk) << 29) | ((uint32_t)q & kMask29);
    const uint32_t P = t0 >> k;
    const uint32_t up = (R > half) || (R == half && (sticky || (P & 1u)));
    o.D = (uint32_t)((R >= half ? R - half : half - R - sticky) >> k);
    o.ybits = (sign << 31) | ((P + up) << k);
    o.dir = up ^ sign;
    return o;
}

// x rounded toward +inf (dir = 1) or -inf (dir = 0) on the same grid
static __host__ __device__ __forceinline__ uint32_t directed_k(uint64_t bits, uint32_t dir, uint32_t k)
{
    const uint32_t hi = (uint32_t)(bits >> 32), lo = (uint32_t)bits;
    const uint32_t sign = hi >> 31, ahi = hi & 0x7FFFFFFFu;
    const uint32_t maskk = (1u << k) - 1u;
    const uint32_t away = dir ^ sign;                                 // rounding grows the magnitude
    if (__builtin_expect(ahi - (897u << 20) < ((2047u - 897u) << 20), 1)) {
        const uint32_t e = ahi - (896u << 20);
        uint32_t t;
        if (__builtin_expect(e >= (255u << 20), 0)) t = away ? kF32Inf : (0x7F7FFFFFu >> k) << k;
        else {
            const uint32_t T = (e << 3) | (lo >> 29);
            const uint32_t inexact = ((T & maskk) | (lo & kMask29)) != 0;
            t = ((T >> k) + (inexact & away)) << k;
        }
        return (sign << 31) | t;
    }
    const uint64_t mag = bits & 0x7FFFFFFFFFFFFFFFull;
    if (mag > 0x7FF0000000000000ull) return kF32QNaN;
    if (mag == 0x7FF0000000000000ull) return (sign << 31) | kF32Inf;
    const uint32_t eb = (uint32_t)(mag >> 52);
    const uint64_t sig = eb ? ((mag & 0x000FFFFFFFFFFFFFull) | (1ull << 52)) : mag;
    const uint32_t sh = eb ? 897u - eb : 896u;
    uint64_t q = 0;
    uint32_t inexact;
    if (sh > 63) { inexact = sig != 0; }
    else { q = sig >> sh; inexact = (sig & ((1ull << sh) - 1)) != 0; }
    const uint32_t t0 = (uint32_t)(q >> 29);
    inexact |= ((t0 & maskk) | ((uint32_t)q & kMask29)) != 0;
    return (sign << 31) | (((t0 >> k) + (inexact & away)) << k);
}

// What every streaming kernel needs of one value: rnd(x), whether it is logged, and the side.
struct Rounded {
    uint32_t ybits;
    bool logged, up;
};

// K0: rounding amount 32 (the hardware conversion does the common case); otherwise k = 32 - b_r.
template <bool K0>
__device__ __forceinline__ Rounded round_decide(double x, uint32_t thr, uint32_t k)
{
    const uint64_t bits = (uint64_t)__double_as_longlong(x);
    Rounded o;
    if (K0) {
        const FastDecision f = decide_fast(x);
        o.ybits = __float_as_uint(f.y);
        o.logged = f.D < thr;
        o.up = f.grow != f.neg;
        // (for +-0 the conversion and D = 2^28 above are already the answer: tensors that are half
        // zeros, as after a ReLU, must not send every wave through the integer path)
        if (__builtin_expect(f.slow, 0)) {
            if (x != 0.0) {
                const Decision d = decide(bits);
                o.ybits = d.ybits; o.logged = d.D < thr; o.up = d.dir != 0;
            }
        }
    } else {
        const Decision d = decide_k(bits, k);
        o.ybits = d.ybits; o.logged = d.D < thr; o.up = d.dir != 0;
    }
    return o;
}

// Monotone integer image of a binary64 pattern (sign-magnitude -> two's complement).
static __host__ __device__ __forceinline__ int64_t ord64(uint64_t bits)
{
    const int64_t mag = (int64_t)(bits & 0x7FFFFFFFFFFFFFFFull);
    return (bits >> 63) ? -mag : mag;
}

__device__ __forceinline__ uint32_t lane_id() { return __lane_id(); }

__device__ __forceinline__ uint32_t popc64(uint64_t v) { return (uint32_t)__popcll(v); }

// number of set bits of m below this lane
__device__ __forceinline__ uint32_t rank_below(uint64_t m)
{
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint64_t ballot(bool p) { return __ballot(p); }

__device__ __forceinline__ uint64_t readlane64(uint64_t v, uint32_t l)
{
    const uint32_t lo = __builtin_amdgcn_readlane((int)(uint32_t)v, (int)l);
    const uint32_t hi = __builtin_amdgcn_readlane((int)(uint32_t)(v >> 32), (int)l);
    return ((uint64_t)hi << 32) | lo;
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// LDS written by some lanes of a wave and read by others of the same wave: LDS operations of
// one wave complete in issue order, so only the compiler has to be kept from reordering.
__device__ __forceinline__ void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

constexpr uint64_t kOneBits = 0x3FF0000000000000ull;   // 1.0: padding value, never logged

// ---- implicit im2col index arithmetic (convolution as GEMM) --------------------------------

// Implicit im2col view of a channels-last image X[N][H][W][C] (A operand modes 2 and 3): the
// matrix element (row m = (n, ho, wo), tap kc = (kh, kw, ci)) is X[n, ho s - p + kh d, wo s - p + kw d, ci],
// zero in the padding.  Indices are split with a reciprocal multiply and one correction step.
struct ConvGeom {
    int32_t H, W, C, Wo, HoWo, KWC;
    int32_t sh, sw, ph, pw, dh, dw;
    int32_t vec;                     // taps (kc, kc + 1), kc even, are one aligned 16-byte load (C even)
    uint32_t rows, taps;             // N Ho Wo and KH KW C
    double inv_HoWo, inv_Wo, inv_KWC, inv_C, inv_sh, inv_sw;
    uint32_t mKWC, mC, msh, msw;     // multipliers of divmod_magic for KWC, C and the strides
    uint32_t mHoWo, mWo;             // and for HoWo and Wo (rows split in scalar registers)
    int32_t uni;                     // the 16 taps of a k step share (kh, kw): C is a multiple of 16
    int32_t Ho, nimg;                // output rows per image, images
    int32_t st_n, st_ho, st_wo;      // kRowStep = st_n HoWo + st_ho Wo + st_wo: one k step of the weight gradient
};

constexpr int kRowStep = 16;         // rows of the image matrix per k step of the transposed view

constexpr int32_t kNowhere = -(1 << 30);        // row / tap coordinate that fails every bounds test

// q = x / d, r = x % d for d >= 1: the double product is within one of the quotient.
static __host__ __device__ __forceinline__ void divmod_u32(uint32_t x, uint32_t d, double inv, uint32_t &q, uint32_t &r)
{
    q = (uint32_t)((double)x * inv);
    int32_t rem = (int32_t)(x - q * d);
    if (rem < 0) { --q; rem += (int32_t)d; }
    else if ((uint32_t)rem >= d) { ++q; rem -= (int32_t)d; }
    r = (uint32_t)rem;
}

// The same split in integer operations only: with m = min(floor(2^32 / d), 2^32 - 1) the high half of
// x m is the quotient or one below it (x / d - x m / 2^32 = x (2^32 - m d) / (d 2^32) < x / 2^32 < 1).
// A wave-uniform x then stays in scalar registers, where the double product above would not.
static __host__ __device__ __forceinline__ void divmod_magic(uint32_t x, uint32_t d, uint32_t m, uint32_t &q, uint32_t &r)
{
    q = (uint32_t)(((uint64_t)x * m) >> 32);
    r = x - q * d;
    if (r >= d) { ++q; r -= d; }
}

static inline uint32_t magic_of(uint32_t d)
{
    const uint64_t m = (1ull << 32) / (d > 0 ? d : 1);
    return m > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)m;
}

struct RowPos { int32_t base, h0, w0, rem; };   // element offset of X[n, h0, w0, 0]; top-left tap position
struct TapPos { int32_t off, hh, ww, rem; };    // (hh W + ww) C + ci with hh = kh dil_h, ww = kw dil_w
// (rem: stride remainders, used by the input-gradient view below only)

// INT: integer-only index split (for a wave-uniform m: the whole row is computed in scalar registers)
template <bool INT = false>
static __host__ __device__ __forceinline__ RowPos conv_row(const ConvGeom &c, uint32_t m)
{
    uint32_t n, rem, ho, wo;
    if (INT) {
        divmod_magic(m, (uint32_t)c.HoWo, c.mHoWo, n, rem);
        divmod_magic(rem, (uint32_t)c.Wo, c.mWo, ho, wo);
    } else {
        divmod_u32(m, (uint32_t)c.HoWo, c.inv_HoWo, n, rem);
        divmod_u32(rem, (uint32_t)c.Wo, c.inv_Wo, ho, wo);
    }
    RowPos r;
    r.h0 = (int32_t)ho * c.sh - c.ph;
    r.w0 = (int32_t)wo * c.sw - c.pw;
    r.base = (int32_t)(((n * (uint32_t)c.H + (uint32_t)r.h0) * (uint32_t)c.W + (uint32_t)r.w0) * (uint32_t)c.C);
    r.rem = 0;
    if (m >= c.rows) r.h0 = kNowhere;
    return r;
}

// A row of the image matrix kept as (n, ho, wo) and moved kRowStep rows at a time (the weight
// gradient walks the rows along k): digit-wise addition with one carry per digit instead of two
// index splits per step.  Walking down adds the complement (Wo - st_wo, Ho - 1 - st_ho, -st_n - 1),
// which lowers the row by kRowStep through the same carries.  Rows before the first or past the
// last image have n outside [0, nimg) and read as padding.
struct RowIter { int32_t n, ho, wo; };

static __host__ __device__ __forceinline__ RowIter row_iter(const ConvGeom &c, uint32_t m)
{
    uint32_t n, rem, ho, wo;
    divmod_u32(m, (uint32_t)c.HoWo, c.inv_HoWo, n, rem);
    divmod_u32(rem, (uint32_t)c.Wo, c.inv_Wo, ho, wo);
    return RowIter{(int32_t)n, (int32_t)ho, (int32_t)wo};
}

static __host__ __device__ __forceinline__ void row_step_digits(const ConvGeom &c, bool down, int32_t &an, int32_t &ah, int32_t &aw)
{
    an = down ? -c.st_n - 1 : c.st_n;
    ah = down ? c.Ho - 1 - c.st_ho : c.st_ho;
    aw = down ? c.Wo - c.st_wo : c.st_wo;
}

static __host__ __device__ __forceinline__ void row_advance(const ConvGeom &c, RowIter &s, int32_t an, int32_t ah, int32_t aw)
{
    s.wo += aw;
    const int32_t cw = s.wo >= c.Wo ? 1 : 0;
    s.wo -= cw ? c.Wo : 0;
    s.ho += ah + cw;
    const int32_t ch = s.ho >= c.Ho ? 1 : 0;
    s.ho -= ch ? c.Ho : 0;
    s.n += an + ch;
}

static __host__ __device__ __forceinline__ RowPos row_pos(const ConvGeom &c, const RowIter &s)
{
    RowPos r;
    const int32_t h0 = s.ho * c.sh - c.ph;
    r.w0 = s.wo * c.sw - c.pw;
    r.base = (int32_t)((((uint32_t)s.n * (uint32_t)c.H + (uint32_t)h0) * (uint32_t)c.W + (uint32_t)r.w0) * (uint32_t)c.C);
    r.h0 = (uint32_t)s.n < (uint32_t)c.nimg ? h0 : kNowhere;
    r.rem = 0;
    return r;
}

// INT: integer-only index split (for a wave-uniform kc: the whole tap is computed in scalar registers)
template <bool INT = false>
static __host__ __device__ __forceinline__ TapPos conv_tap(const ConvGeom &c, uint32_t kc)
{
    uint32_t kh, rem, kw, ci;
    if (INT) {
        divmod_magic(kc, (uint32_t)c.KWC, c.mKWC, kh, rem);
        divmod_magic(rem, (uint32_t)c.C, c.mC, kw, ci);
    } else {
        divmod_u32(kc, (uint32_t)c.KWC, c.inv_KWC, kh, rem);
        divmod_u32(rem, (uint32_t)c.C, c.inv_C, kw, ci);
    }
    TapPos t;
    t.hh = (int32_t)kh * c.dh;
    t.ww = (int32_t)kw * c.dw;
    t.off = (int32_t)(((uint32_t)t.hh * (uint32_t)c.W + (uint32_t)t.ww) * (uint32_t)c.C + ci);
    t.rem = 0;
    if (kc >= c.taps) t.hh = kNowhere;
    return t;
}

// Input gradient (A operand mode 4).  The gathered image is dY[N][Ho][Wo][Cout]; matrix row
// m = (n, h, w) is a position of the layer's input, column kc = (kh, kw, co), and the element is
// dY[n, ho, wo, co] for the output position with ho s - p + kh d = h (likewise in w): zero when
// h + p - kh d is not a multiple of the stride or ho falls outside the output.  With
// h + p = s qh + rh and kh d = s qk + rk (remainders in [0, s)), the difference is a multiple of s
// exactly when rh = rk, and then ho = qh - qk: the address splits into a row part and a tap part
// as in the forward view.  The geometry reuses ConvGeom with the roles exchanged: (H, W, C) are
// dY's (Ho, Wo, Cout); (Wo, HoWo) the input's (W, H W); KWC = KW Cout; rows = N H W; taps = KH KW Cout.
static __host__ __device__ __forceinline__ RowPos dgrad_row(const ConvGeom &c, uint32_t m)
{
    uint32_t n, rem, h, w;
    divmod_u32(m, (uint32_t)c.HoWo, c.inv_HoWo, n, rem);
    divmod_u32(rem, (uint32_t)c.Wo, c.inv_Wo, h, w);
    const uint32_t hp = h + (uint32_t)c.ph, wp = w + (uint32_t)c.pw;
    const uint32_t qh = hp / (uint32_t)c.sh, qw = wp / (uint32_t)c.sw;           // once per row and thread
    RowPos r;
    r.h0 = (int32_t)qh;
    r.w0 = (int32_t)qw;
    r.rem = (int32_t)((hp - qh * (uint32_t)c.sh) | ((wp - qw * (uint32_t)c.sw) << 16));
    r.base = (int32_t)(((n * (uint32_t)c.H + qh) * (uint32_t)c.W + qw) * (uint32_t)c.C);
    if (m >= c.rows) r.h0 = kNowhere;
    return r;
}

template <bool INT = false>
static __host__ __device__ __forceinline__ TapPos dgrad_tap(const ConvGeom &c, uint32_t kc)
{
    uint32_t kh, rem, kw, co, qk, rk, qkw, rkw;
    if (INT) {
        divmod_magic(kc, (uint32_t)c.KWC, c.mKWC, kh, rem);
        divmod_magic(rem, (uint32_t)c.C, c.mC, kw, co);
        divmod_magic(kh * (uint32_t)c.dh, (uint32_t)c.sh, c.msh, qk, rk);
        divmod_magic(kw * (uint32_t)c.dw, (uint32_t)c.sw, c.msw, qkw, rkw);
    } else {
        divmod_u32(kc, (uint32_t)c.KWC, c.inv_KWC, kh, rem);
        divmod_u32(rem, (uint32_t)c.C, c.inv_C, kw, co);
        divmod_u32(kh * (uint32_t)c.dh, (uint32_t)c.sh, c.inv_sh, qk, rk);
        divmod_u32(kw * (uint32_t)c.dw, (uint32_t)c.sw, c.inv_sw, qkw, rkw);
    }
    TapPos t;
    t.hh = -(int32_t)qk;
    t.ww = -(int32_t)qkw;
    t.rem = (int32_t)(rk | (rkw << 16));
    t.off = (int32_t)(co - (qk * (uint32_t)c.W + qkw) * (uint32_t)c.C);
    if (kc >= c.taps) t.hh = kNowhere;
    return t;
}


static inline ConvGeom conv_geom(int64_t N, int64_t H, int64_t W, int64_t C, int64_t KH, int64_t KW, int64_t sh,
                                 int64_t sw, int64_t ph, int64_t pw, int64_t dh, int64_t dw, int64_t Ho, int64_t Wo,
                                 bool vec)
{
    ConvGeom c;
    c.H = (int32_t)H; c.W = (int32_t)W; c.C = (int32_t)C; c.Wo = (int32_t)Wo;
    c.HoWo = (int32_t)(Ho * Wo); c.KWC = (int32_t)(KW * C);
    c.sh = (int32_t)sh; c.sw = (int32_t)sw; c.ph = (int32_t)ph; c.pw = (int32_t)pw; c.dh = (int32_t)dh; c.dw = (int32_t)dw;
    c.vec = vec ? 1 : 0;
    c.rows = (uint32_t)(N * Ho * Wo); c.taps = (uint32_t)(KH * KW * C);
    c.Ho = (int32_t)Ho; c.nimg = (int32_t)N;
    {
        const int64_t hw = Ho * Wo > 0 ? Ho * Wo : 1, wq = Wo > 0 ? Wo : 1;
        c.st_n = (int32_t)(kRowStep / hw); c.st_ho = (int32_t)(kRowStep % hw / wq); c.st_wo = (int32_t)(kRowStep % hw % wq);
    }
    c.inv_HoWo = 1.0 / (double)(c.HoWo > 0 ? c.HoWo : 1); c.inv_Wo = 1.0 / (double)(c.Wo > 0 ? c.Wo : 1);
    c.inv_KWC = 1.0 / (double)(c.KWC > 0 ? c.KWC : 1); c.inv_C = 1.0 / (double)(c.C > 0 ? c.C : 1);
    c.inv_sh = 1.0 / (double)c.sh; c.inv_sw = 1.0 / (double)c.sw;
    c.mKWC = magic_of((uint32_t)c.KWC); c.mC = magic_of((uint32_t)c.C);
    c.msh = magic_of((uint32_t)c.sh); c.msw = magic_of((uint32_t)c.sw);
    c.mHoWo = magic_of((uint32_t)c.HoWo); c.mWo = magic_of((uint32_t)c.Wo);
    c.uni = vec && c.C > 0 && c.C % 16 == 0 ? 1 : 0;
    return c;
}

// The same structure for the input-gradient view of a layer with input (N, H, W, C), output
// (N, Ho, Wo, Cout): see dgrad_row.
static inline ConvGeom dgrad_geom(int64_t N, int64_t H, int64_t W, int64_t Cout, int64_t KH, int64_t KW, int64_t sh,
                                  int64_t sw, int64_t ph, int64_t pw, int64_t dh, int64_t dw, int64_t Ho, int64_t Wo,
                                  bool vec)
{
    ConvGeom c;
    c.H = (int32_t)Ho; c.W = (int32_t)Wo; c.C = (int32_t)Cout; c.Wo = (int32_t)W;
    c.HoWo = (int32_t)(H * W); c.KWC = (int32_t)(KW * Cout);
    c.sh = (int32_t)sh; c.sw = (int32_t)sw; c.ph = (int32_t)ph; c.pw = (int32_t)pw; c.dh = (int32_t)dh; c.dw = (int32_t)dw;
    c.vec = vec ? 1 : 0;
    c.rows = (uint32_t)(N * H * W); c.taps = (uint32_t)(KH * KW * Cout);
    c.Ho = (int32_t)H; c.nimg = (int32_t)N; c.st_n = c.st_ho = c.st_wo = 0;      // (rows are not walked along k in this view)
    c.inv_HoWo = 1.0 / (double)(c.HoWo > 0 ? c.HoWo : 1); c.inv_Wo = 1.0 / (double)(c.Wo > 0 ? c.Wo : 1);
    c.inv_KWC = 1.0 / (double)(c.KWC > 0 ? c.KWC : 1); c.inv_C = 1.0 / (double)(c.C > 0 ? c.C : 1);
    c.inv_sh = 1.0 / (double)c.sh; c.inv_sw = 1.0 / (double)c.sw;
    c.mKWC = magic_of((uint32_t)c.KWC); c.mC = magic_of((uint32_t)c.C);
    c.msh = magic_of((uint32_t)c.sh); c.msw = magic_of((uint32_t)c.sw);
    c.mHoWo = magic_of((uint32_t)c.HoWo); c.mWo = magic_of((uint32_t)c.Wo);
    c.uni = vec && c.C > 0 && c.C % 16 == 0 ? 1 : 0;
    return c;
}

// Element offset of the im2col matrix entry (row m, tap kc) in the image, or -1 when it is a
// padding zero or lies outside the matrix: what conv_gather loads, as one function.
template <bool INT = false>
static __host__ __device__ __forceinline__ int64_t conv_element(const ConvGeom &c, uint32_t m, uint32_t kc)
{
    const RowPos r = conv_row(c, m);
    const TapPos t = conv_tap<INT>(c, kc);
    const bool ok = (uint32_t)(r.h0 + t.hh) < (uint32_t)c.H && (uint32_t)(r.w0 + t.ww) < (uint32_t)c.W;
    return ok ? (int64_t)(r.base + t.off) : -1;
}

// The same for the input-gradient view: offset into dY of matrix entry (row m, column kc), or -1.
template <bool INT = false>
static __host__ __device__ __forceinline__ int64_t dgrad_element(const ConvGeom &c, uint32_t m, uint32_t kc)
{
    const RowPos r = dgrad_row(c, m);
    const TapPos t = dgrad_tap<INT>(c, kc);
    const bool ok = (uint32_t)(r.h0 + t.hh) < (uint32_t)c.H && (uint32_t)(r.w0 + t.ww) < (uint32_t)c.W && r.rem == t.rem;
    return ok ? (int64_t)(r.base + t.off) : -1;
}

}  // namespace vt
