// vt_conv_phases.h -- input gradient of a strided convolution as one small GEMM per stride phase.
//
// For a layer with stride s the term dY[n,ho,wo,co] W[kh,kw,ci,co] reaches input position h only
// when h + p - kh d = s ho, so an input position with (h + p) mod s = a receives contributions
// from the filter rows with (kh d) mod s = a alone: in the single-GEMM view of the gradient all
// other entries of its row are zeros (3 of 4 at stride 2).  Splitting the input positions by
// their phase (a, b) = ((h + p) mod s_h, (w + p) mod s_w) gives s_h s_w independent problems,
// each a stride-1 gradient over the sub-grid h = s q + a - p with the sub-filter of its phase,
// none of which multiplies a structural zero:
//     ho = q - qk,   q = q0 + i  (i = 0 .. Ha-1),   kh_t = kh0 + st t,   qk_t = (kh_t d - a) / s = qk0 + dq t
// which is the stride-1 geometry with padding q0 - qk0 (it may be negative) and dilation dq.
// Host code only; the kernels see each phase as an ordinary geometry.
#pragma once
#include <stdint.h>

namespace vt {

struct PhaseAxis {         // one phase along one axis
    int64_t q0 = 0;        // first q with s q + a - p >= 0
    int64_t count = 0;     // input positions of this phase (Ha)
    int64_t k0 = 0;        // first filter index of the phase
    int64_t kstep = 1;     // distance between the phase's filter indices
    int64_t taps = 0;      // filter indices in the phase
    int64_t pad = 0;       // padding of the stride-1 sub-problem: q0 - qk0
    int64_t dil = 1;       // its dilation: dq
};

// Phase a of an axis: input size `size`, filter size `K`, stride s, padding p, dilation d.
static inline PhaseAxis phase_axis(int64_t size, int64_t K, int64_t s, int64_t p, int64_t d, int64_t a)
{
    PhaseAxis x;
    x.q0 = p > a ? (p - a + s - 1) / s : 0;
    const int64_t top = size - 1 + p - a;                       // s q <= top
    x.count = top < 0 ? 0 : top / s - x.q0 + 1;
    if (x.count < 0) x.count = 0;
    int64_t second = -1;
    for (int64_t k = 0; k < K; ++k)
        if ((k * d) % s == a) {
            if (x.taps == 0) x.k0 = k;
            else if (x.taps == 1) second = k;
            ++x.taps;
        }
    x.kstep = second >= 0 ? second - x.k0 : 1;
    const int64_t qk0 = x.taps ? (x.k0 * d - a) / s : 0;
    x.dil = x.taps > 1 ? (x.kstep * d) / s : 1;
    x.pad = x.q0 - qk0;
    return x;
}

}  // namespace vt
