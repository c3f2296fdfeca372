// vt_source.h -- where the FP64 values of the streaming trainer kernels come from: a tensor in
// memory, or an element-wise / row-wise layer evaluated on the fly so that its FP64 output never
// goes to memory (residual add, ReLU, GELU, layer norm, softmax: the non-GEMM layers of a
// transformer block, each an "intermediate computation" whose output the method rounds).
#pragma once
#include "vt_device.h"
#include "vt_kernels.h"

#include <math.h>

namespace vt {

typedef double src_d2 __attribute__((ext_vector_type(2)));

// An FP64 tensor in memory.  pair(e) returns elements e and e + 1; past the end it returns 1.0,
// a value that is never logged.
struct PlainSource {
    const double *x;
    template <bool FULL, bool VEC>
    __device__ __forceinline__ src_d2 pair(uint64_t e, uint64_t n) const
    {
        src_d2 v;
        if (VEC && (FULL || e + 1 < n)) v = __builtin_nontemporal_load((const src_d2 *)(x + e));
        else {
            v.x = e < n ? x[e] : 1.0;
            v.y = e + 1 < n ? x[e + 1] : 1.0;
        }
        return v;
    }
    template <bool FULL, bool VEC>
    __device__ __forceinline__ void keep(uint64_t, uint64_t, src_d2) const {}
};

// The result of a split-K GEMM before its single rounding: the K slices' partial sums (slabs of
// `slab` doubles, slab even, 16-byte aligned) added in ascending (variant 0) or descending slice
// order, scaled and biased -- alpha * (P0 + P1 + ...) + bias[column] -- evaluated where the
// trainer hook consumes it, so the sum never goes to memory (unless y64 asks for a copy).
struct SplitKSource {
    const double *P;
    uint64_t slab;
    int splits, variant;
    double alpha;
    const double *bias;       // per output column, or null
    uint32_t ncols;
    double inv_ncols;
    double *y64;
    template <bool FULL, bool VEC>
    __device__ __forceinline__ src_d2 pair(uint64_t e, uint64_t n) const
    {
        const bool has0 = FULL || e < n, has1 = FULL || e + 1 < n;
        src_d2 acc = {0.0, 0.0};
        if (has0) {
            auto slice = [&](int k) {
                const double *p = P + (uint64_t)(variant ? splits - 1 - k : k) * slab + e;
                src_d2 v;
                if (has1) v = *(const src_d2 *)p;
                else { v.x = p[0]; v.y = 0.0; }
                return v;
            };
            int k = 0;
            for (; k + 4 <= splits; k += 4) {                 // four loads in flight, additions still in order
                const src_d2 v0 = slice(k), v1 = slice(k + 1), v2 = slice(k + 2), v3 = slice(k + 3);
                acc.x = acc.x + v0.x; acc.y = acc.y + v0.y;
                acc.x = acc.x + v1.x; acc.y = acc.y + v1.y;
                acc.x = acc.x + v2.x; acc.y = acc.y + v2.y;
                acc.x = acc.x + v3.x; acc.y = acc.y + v3.y;
            }
            for (; k < splits; ++k) {
                const src_d2 v = slice(k);
                acc.x = acc.x + v.x; acc.y = acc.y + v.y;
            }
        }
        src_d2 c;
        c.x = alpha * acc.x;
        c.y = alpha * acc.y;
        if (bias && has0) {
            uint32_t r, c0;
            divmod_u32((uint32_t)e, ncols, inv_ncols, r, c0);
            const uint32_t c1 = c0 + 1u == ncols ? 0u : c0 + 1u;
            c.x = c.x + bias[c0];
            if (has1) c.y = c.y + bias[c1];
        }
        if (!has0) c.x = 1.0;
        if (!has1) c.y = 1.0;
        return c;
    }
    template <bool FULL, bool VEC>
    __device__ __forceinline__ void keep(uint64_t e, uint64_t n, src_d2 v) const
    {
        if (!y64) return;
        if (FULL || e + 1 < n) *(src_d2 *)(y64 + e) = v;
        else if (e < n) y64[e] = v.x;
    }
};

// The input gradient of a strided convolution computed phase by phase (strides 1 or 2 per axis):
// the positions (n, h, w) of the layer's input with ((h + p_h) mod s_h, (w + p_w) mod s_w) = (a, b)
// form a dense sub-grid whose FP64 results lie in slab (a, b), rows (n, i, j) by C channels.
// Element e of the gradient [N][H][W][C] is looked up in its slab; a phase that no filter tap
// reaches has no slab and reads as zero.  C is even, so a pair (e, e + 1) shares its position.
struct PhaseSource {
    const double *P;
    uint32_t C, W, HW;
    double inv_C, inv_W, inv_HW;
    uint32_t ph, pw, shift_h, shift_w;     // shift = stride - 1 (0 or 1): phase = low bit, q = the rest
    uint32_t q0h[2], Ha[2], q0w[2], Wb[2];
    uint32_t off[4];                       // first element of slab (a, b) at off[2 a + b]
    uint32_t has;                          // bit 2 a + b: the phase has a slab
    double *y64;
    template <bool FULL, bool VEC>
    __device__ __forceinline__ src_d2 pair(uint64_t e, uint64_t n) const
    {
        src_d2 v = {1.0, 1.0};
        if (!(FULL || e + 1 < n)) {
            if (e < n) v.x = one((uint32_t)e);
            return v;
        }
        uint32_t pos, c, img, rem, h, w;
        divmod_u32((uint32_t)e, C, inv_C, pos, c);
        divmod_u32(pos, HW, inv_HW, img, rem);
        divmod_u32(rem, W, inv_W, h, w);
        const uint32_t hp = h + ph, wp = w + pw;
        const uint32_t a = hp & shift_h, b = wp & shift_w;
        const uint32_t i = (hp >> shift_h) - (a ? q0h[1] : q0h[0]), j = (wp >> shift_w) - (b ? q0w[1] : q0w[0]);
        const uint32_t rows_h = a ? Ha[1] : Ha[0], rows_w = b ? Wb[1] : Wb[0];
        const uint32_t o = a ? (b ? off[3] : off[2]) : (b ? off[1] : off[0]);
        const bool live = (has >> (2u * a + b)) & 1u;
        const uint32_t at = live ? o + ((img * rows_h + i) * rows_w + j) * C + c : 0u;
        const src_d2 x = *(const src_d2 *)(P + at);
        v.x = live ? x.x : 0.0;
        v.y = live ? x.y : 0.0;
        return v;
    }
    __device__ __forceinline__ double one(uint32_t e) const      // a single element (odd tail; not reached for even C)
    {
        uint32_t pos, c, img, rem, h, w;
        divmod_u32(e, C, inv_C, pos, c);
        divmod_u32(pos, HW, inv_HW, img, rem);
        divmod_u32(rem, W, inv_W, h, w);
        const uint32_t hp = h + ph, wp = w + pw;
        const uint32_t a = hp & shift_h, b = wp & shift_w;
        const uint32_t i = (hp >> shift_h) - (a ? q0h[1] : q0h[0]), j = (wp >> shift_w) - (b ? q0w[1] : q0w[0]);
        const uint32_t rows_h = a ? Ha[1] : Ha[0], rows_w = b ? Wb[1] : Wb[0];
        const uint32_t o = a ? (b ? off[3] : off[2]) : (b ? off[1] : off[0]);
        const bool live = (has >> (2u * a + b)) & 1u;
        return live ? P[o + ((img * rows_h + i) * rows_w + j) * C + c] : 0.0;
    }
    template <bool FULL, bool VEC>
    __device__ __forceinline__ void keep(uint64_t e, uint64_t n, src_d2 v) const
    {
        if (!y64) return;
        if (FULL || e + 1 < n) *(src_d2 *)(y64 + e) = v;
        else if (e < n) y64[e] = v.x;
    }
};

// One output of an element-wise layer from its input value(s).
template <int OP>
__device__ __forceinline__ double layer_value(double xa, double xb)
{
    switch (OP) {                                                     // compile-time
    case kLayerAdd: return xa + xb;
    case kLayerRelu: return xa > 0.0 ? xa : (xa != xa ? xa : 0.0);
    case kLayerGeluTanh: {
        // x/2 (1 + tanh u) = x / (1 + exp(-2u)): the same function with one exponential, no
        // cancellation anywhere, and the right limits (0 for very negative x, x for large x)
        const double x3 = xa * xa * xa;
        const double u = 0.7978845608028654 * (xa + 0.044715 * x3);   // sqrt(2 / pi)
        return xa / (1.0 + exp(-2.0 * u));
    }
    default: return 0.5 * xa * (1.0 + erf(xa * 0.7071067811865476));   // kLayerGeluErf
    }
}

// One output of a row-wise layer from its row statistics st = (mean, 1/std) or (max, 1/sum).
template <int OP>
__device__ __forceinline__ double row_value(const LayerArgs &g, uint32_t r, uint32_t c, double xa, src_d2 st)
{
    if (OP == kLayerNorm) {
        double v = (xa - st.x) * st.y;
        if (g.gamma) v = v * g.gamma[c];
        if (g.beta) v = v + g.beta[c];
        return v;
    }
    uint32_t seen = g.cols;
    if (g.period) {
        uint32_t q, rem;
        divmod_u32(r, g.period, g.inv_period, q, rem);
        seen = rem + 1u < g.cols ? rem + 1u : g.cols;
    }
    return c < seen ? exp(g.scale * xa - st.x) * st.y : 0.0;
}

// One output of batch norm from its column statistics st = (mean, 1/std).
template <int OP>
__device__ __forceinline__ double col_value(const LayerArgs &g, uint32_t c, double xa, src_d2 st)
{
    double v = (xa - st.x) * st.y;
    if (g.gamma) v = v * g.gamma[c];
    if (g.beta) v = v + g.beta[c];
    if (OP == kLayerBatchNormRelu) v = v > 0.0 ? v : (v != v ? v : 0.0);
    return v;
}

template <int OP>
struct LayerSource {
    LayerArgs g;
    template <bool FULL, bool VEC>
    __device__ __forceinline__ src_d2 pair(uint64_t e, uint64_t n) const
    {
        const src_d2 xa = PlainSource{g.a}.template pair<FULL, VEC>(e, n);
        if (OP >= kLayerBatchNorm) {
            // statistics are per column: indices past the end are clamped, their values replaced below
            uint32_t r0, c0;
            divmod_u32((uint32_t)(FULL || e < n ? e : n - 1), g.cols, g.inv_cols, r0, c0);
            const uint32_t c1 = (FULL || e + 1 < n) ? (c0 + 1u == g.cols ? 0u : c0 + 1u) : c0;
            src_d2 v;
            v.x = col_value<OP>(g, c0, xa.x, *(const src_d2 *)(g.stat + 2 * (uint64_t)c0));
            v.y = col_value<OP>(g, c1, xa.y, *(const src_d2 *)(g.stat + 2 * (uint64_t)c1));
            if (!FULL) {
                if (e >= n) v.x = 1.0;
                if (e + 1 >= n) v.y = 1.0;
            }
            return v;
        }
        if (OP == kLayerNorm || OP == kLayerSoftmax) {
            // split the index once, one 16-byte load of the row statistics (a second one only when
            // the pair straddles two rows); indices past the end are clamped to the last output so
            // that the statistics they select exist, and their values replaced below
            uint32_t r0, c0;
            divmod_u32((uint32_t)(FULL || e < n ? e : n - 1), g.cols, g.inv_cols, r0, c0);
            const bool has1 = FULL || e + 1 < n;
            const bool wrap = has1 && c0 + 1u == g.cols;
            const uint32_t r1 = wrap ? r0 + 1u : r0, c1 = has1 ? (wrap ? 0u : c0 + 1u) : c0;
            const src_d2 s0 = *(const src_d2 *)(g.stat + 2 * (uint64_t)r0);
            src_d2 s1 = s0;
            if (wrap) s1 = *(const src_d2 *)(g.stat + 2 * (uint64_t)r1);
            src_d2 v;
            v.x = row_value<OP>(g, r0, c0, xa.x, s0);
            v.y = row_value<OP>(g, r1, c1, xa.y, s1);
            if (!FULL) {
                if (e >= n) v.x = 1.0;
                if (e + 1 >= n) v.y = 1.0;
            }
            return v;
        }
        src_d2 xb = {0.0, 0.0};
        if (OP == kLayerAdd) xb = PlainSource{g.b}.template pair<FULL, VEC>(e, n);
        src_d2 v;
        v.x = layer_value<OP>(xa.x, xb.x);
        v.y = layer_value<OP>(xa.y, xb.y);
        if (!FULL) {
            if (e >= n) v.x = 1.0;
            if (e + 1 >= n) v.y = 1.0;
        }
        return v;
    }
    template <bool FULL, bool VEC>
    __device__ __forceinline__ void keep(uint64_t e, uint64_t n, src_d2 v) const
    {
        if (!g.y64) return;
        if (VEC && (FULL || e + 1 < n)) *(src_d2 *)(g.y64 + e) = v;
        else {
            if (e < n) g.y64[e] = v.x;
            if (e + 1 < n) g.y64[e + 1] = v.y;
        }
    }
};

}  // namespace vt
