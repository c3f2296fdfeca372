// Test helper: runs the library's per-element integer arithmetic (csrc/vt_device.h) on the HOST
// CPU, so its rounding / distance / direction logic can be compared with the oracle without a GPU.
#include "../paper_2403_09603_amd/csrc/vt_device.h"
#include "../paper_2403_09603_amd/csrc/vt_conv_phases.h"
extern "C" void h_decide(const uint64_t *bits, uint64_t n, uint32_t *y, uint32_t *D, uint32_t *dir)
{
    for (uint64_t i = 0; i < n; ++i) {
        vt::Decision d = vt::decide(bits[i]);
        y[i] = d.ybits; D[i] = d.D; dir[i] = d.dir;
    }
}
extern "C" void h_directed(const uint64_t *bits, uint64_t n, uint32_t dir, uint32_t *y)
{
    for (uint64_t i = 0; i < n; ++i) y[i] = vt::directed(bits[i], dir);
}

extern "C" void h_decide_k(const uint64_t *bits, uint64_t n, uint32_t k, uint32_t *y, uint32_t *D, uint32_t *dir)
{
    for (uint64_t i = 0; i < n; ++i) {
        vt::Decision d = vt::decide_k(bits[i], k);
        y[i] = d.ybits; D[i] = d.D; dir[i] = d.dir;
    }
}
extern "C" void h_directed_k(const uint64_t *bits, uint64_t n, uint32_t dir, uint32_t k, uint32_t *y)
{
    for (uint64_t i = 0; i < n; ++i) y[i] = vt::directed_k(bits[i], dir, k);
}

// im2col index arithmetic of the convolution loader: offsets[m * taps + kc] = image element or -1
extern "C" void h_im2col_offsets(const int64_t *g /* N H W C KH KW sh sw ph pw dh dw Ho Wo */, uint32_t row0, uint32_t rows_to_do,
                                 uint32_t tap0, uint32_t taps_to_do, int64_t *offsets)
{
    const vt::ConvGeom c = vt::conv_geom(g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10], g[11], g[12],
                                         g[13], false);
    for (uint32_t m = 0; m < rows_to_do; ++m)
        for (uint32_t k = 0; k < taps_to_do; ++k) offsets[(uint64_t)m * taps_to_do + k] = vt::conv_element(c, row0 + m, tap0 + k);
}

// the input-gradient view of the same loader: offsets[m * cols + kc] = element of dY or -1
extern "C" void h_dgrad_offsets(const int64_t *g /* N H W Cout KH KW sh sw ph pw dh dw Ho Wo */, uint32_t row0, uint32_t rows_to_do,
                                uint32_t col0, uint32_t cols_to_do, int64_t *offsets)
{
    const vt::ConvGeom c = vt::dgrad_geom(g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10], g[11], g[12],
                                          g[13], false);
    for (uint32_t m = 0; m < rows_to_do; ++m)
        for (uint32_t k = 0; k < cols_to_do; ++k) offsets[(uint64_t)m * cols_to_do + k] = vt::dgrad_element(c, row0 + m, col0 + k);
}

// The integer-only index split (used where the tap is wave-uniform): quotient and remainder for given
// (x, d), and the number of (row, tap) pairs on which the two forms of the loader's arithmetic disagree.
extern "C" void h_divmod_magic(const uint32_t *x, const uint32_t *d, uint64_t n, uint32_t *q, uint32_t *r)
{
    for (uint64_t i = 0; i < n; ++i) vt::divmod_magic(x[i], d[i], vt::magic_of(d[i]), q[i], r[i]);
}

extern "C" uint64_t h_tap_split_mismatches(const int64_t *g /* N H W C|Cout KH KW sh sw ph pw dh dw Ho Wo */, int dgrad,
                                           uint32_t row0, uint32_t rows_to_do)
{
    const vt::ConvGeom c = dgrad ? vt::dgrad_geom(g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10], g[11],
                                                  g[12], g[13], false)
                                 : vt::conv_geom(g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10], g[11],
                                                 g[12], g[13], false);
    uint64_t bad = 0;
    for (uint32_t m = row0; m < row0 + rows_to_do; ++m)
        for (uint32_t k = 0; k < c.taps + 40; ++k)
            bad += dgrad ? vt::dgrad_element<true>(c, m, k) != vt::dgrad_element<false>(c, m, k)
                         : vt::conv_element<true>(c, m, k) != vt::conv_element<false>(c, m, k);
    return bad;
}

// The weight gradient's row walk: from row m0, `steps` moves of kRowStep rows up or down; the number
// of positions at which the walked row differs from the directly split one (rows outside the matrix
// must read as padding, whatever their digits are).
extern "C" uint64_t h_row_walk_mismatches(const int64_t *g /* N H W C KH KW sh sw ph pw dh dw Ho Wo */, uint32_t m0, uint32_t steps, int down)
{
    const vt::ConvGeom c = vt::conv_geom(g[0], g[1], g[2], g[3], g[4], g[5], g[6], g[7], g[8], g[9], g[10], g[11], g[12],
                                         g[13], false);
    vt::RowIter it = vt::row_iter(c, m0);
    int32_t an, ah, aw;
    vt::row_step_digits(c, down != 0, an, ah, aw);
    uint64_t bad = 0;
    for (uint32_t i = 0; i <= steps; ++i) {
        const int64_t m = (int64_t)m0 + (down ? -1 : 1) * (int64_t)vt::kRowStep * i;
        const vt::RowPos got = vt::row_pos(c, it);
        if (m < 0 || m >= (int64_t)c.rows) bad += got.h0 != vt::kNowhere;
        else {
            const vt::RowPos want = vt::conv_row(c, (uint32_t)m);
            bad += got.h0 != want.h0 || got.w0 != want.w0 || got.base != want.base || got.rem != want.rem;
        }
        vt::row_advance(c, it, an, ah, aw);
    }
    return bad;
}

// One stride phase of the input gradient, planned and indexed as the library does it: the phase's
// axes go to info[0..13] (q0, count, k0, kstep, taps, pad, dil for h, then for w) and
// offsets[m * cols + kc] = element of dY that the phase's GEMM reads at (row m, column kc), or -1.
extern "C" void h_dgrad_phase_offsets(const int64_t *g /* N H W Cout KH KW sh sw ph pw dh dw Ho Wo */, int64_t a, int64_t b,
                                      uint32_t row0, uint32_t rows_to_do, uint32_t col0, uint32_t cols_to_do,
                                      int64_t *info, int64_t *offsets)
{
    const vt::PhaseAxis ax = vt::phase_axis(g[1], g[4], g[6], g[8], g[10], a);
    const vt::PhaseAxis bx = vt::phase_axis(g[2], g[5], g[7], g[9], g[11], b);
    const vt::PhaseAxis *axes[2] = {&ax, &bx};
    for (int i = 0; i < 2; ++i) {
        int64_t *o = info + 7 * i;
        o[0] = axes[i]->q0; o[1] = axes[i]->count; o[2] = axes[i]->k0; o[3] = axes[i]->kstep; o[4] = axes[i]->taps;
        o[5] = axes[i]->pad; o[6] = axes[i]->dil;
    }
    const vt::ConvGeom c = vt::dgrad_geom(g[0], ax.count, bx.count, g[3], ax.taps, bx.taps, 1, 1, ax.pad, bx.pad, ax.dil, bx.dil,
                                          g[12], g[13], false);
    for (uint32_t m = 0; m < rows_to_do; ++m)
        for (uint32_t k = 0; k < cols_to_do; ++k) offsets[(uint64_t)m * cols_to_do + k] = vt::dgrad_element(c, row0 + m, col0 + k);
}

// SHA-256 of one byte range with the library's per-lane routines (csrc/vt_sha256.h), stepping
// through the blocks the way the chunk kernel does: whole blocks, then the ragged end or the
// constant padding block.
#include "../paper_2403_09603_amd/csrc/vt_sha256.h"
extern "C" void h_sha256(const uint8_t *data, uint64_t len, uint8_t *digest)
{
    vt::Sha256State s;
    vt::sha256_init(s);
    const uint64_t blocks = len >> 6;
    for (uint64_t b = 0; b < blocks; ++b) {
        uint32_t w[16];
        for (int i = 0; i < 16; ++i) {
            uint32_t v;
            __builtin_memcpy(&v, data + 64 * b + 4 * i, 4);
            w[i] = vt::sha_bswap(v);
        }
        vt::sha256_compress(s, w);
    }
    const uint32_t rem = (uint32_t)(len & 63);
    if (rem) vt::sha256_finish_ragged(s, data + 64 * blocks, rem, len);
    else vt::sha256_pad_block(s, len);
    for (int i = 0; i < 8; ++i) {
        const uint32_t v = vt::sha_bswap(s.h[i]);
        __builtin_memcpy(digest + 4 * i, &v, 4);
    }
}

// the GEMM epilogue's form of the threshold test: (r - c0) <u c1 on the 29 dropped bits
extern "C" void h_window_test(const uint32_t *r, uint64_t n, uint32_t thr, uint8_t *logged)
{
    const uint32_t c0 = vt::thr_window_base(thr), c1 = vt::thr_window_size(thr);
    for (uint64_t i = 0; i < n; ++i) logged[i] = (uint8_t)(((r[i] & vt::kMask29) - c0) < c1);
}

// and its shifted form on whole low words (any upper three bits)
extern "C" void h_window_key_test(const uint32_t *lo, uint64_t n, uint32_t thr, uint8_t *logged)
{
    const uint32_t nbase = 0u - vt::thr_window_base(thr), size_s = vt::thr_window_size(thr) << 3;
    for (uint64_t i = 0; i < n; ++i) logged[i] = (uint8_t)(vt::window_key(lo[i], nbase) < size_s);
}
