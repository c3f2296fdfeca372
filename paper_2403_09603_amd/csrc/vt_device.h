// vt_device.h -- per-element device arithmetic of the round/log/replay path (gfx950).
//
// Everything here works on the binary64 bit pattern with integer instructions only, so the
// result does not depend on the wave's rounding or denormal MODE bits.
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
// Lanes with slow == true must be redone with decide() (NaN, Inf, zero, tiny, |x| >= 2^128).
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

}  // namespace vt
