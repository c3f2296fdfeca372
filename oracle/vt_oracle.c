/*
 * vt_oracle.c -- plain CPU oracle (test infrastructure only; see vt_oracle.h).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC vt_oracle.c -lm
 * Every floating-point step below is exact or a single IEEE operation; nothing here is
 * blocked, fused or reordered beyond what the paper's algorithms state.
 */
#include "vt_oracle.h"

#include <math.h>
#include <string.h>

static uint64_t f64_bits(double x) { uint64_t b; memcpy(&b, &x, 8); return b; }
static uint32_t f32_bits(float x)  { uint32_t b; memcpy(&b, &x, 4); return b; }
static float    f32_from(uint32_t b) { float x; memcpy(&x, &b, 4); return x; }

#define TWO28 268435456.0 /* 2^28 */

/* Method, primitive 1 with b_r = 32: "round to the nearest FP32".  The C conversion from
 * double to float under the default rounding mode IS the IEEE convertFormat operation with
 * roundTiesToEven, so the definition is the cast itself. */
static float rnd32(double x) { return (float)x; }

/* Method, primitive 1 for b_r < 32 (and the caption of the floating-point figure): the nearest
 * 32-bit float that has zeros in the last 32 - b_r bits of its mantissa, i.e. the nearest point
 * of the grid with b_r - 9 mantissa bits in x's binade (spacing 2^(32 - b_r) ulp32).  Written
 * with exact binary64 steps: scale so that the grid becomes the integers, round to the nearest
 * integer with ties to even (rint under the default mode), scale back.  Below 2^-126 the FP32
 * spacing is fixed at 2^-149, so the grid is the multiples of 2^(-149 + 32 - b_r).  A result of
 * 2^128 or more is infinity.  b_r = 32 is the cast above. */
static int valid_br(int b_r) { return b_r >= 10 && b_r <= 32; }

static int grid_scale_exponent(double x, int b_r)      /* grid spacing at x is 2^(-this) */
{
    int E = ilogb(x);
    if (E < -126) E = -126;
    return (b_r - 9) - E;
}

static float rnd_b(double x, int b_r)
{
    if (b_r == 32) return rnd32(x);
    if (isnan(x) || isinf(x) || x == 0.0) return (float)x;
    int sc = grid_scale_exponent(x, b_r);
    double y = scalbn(rint(scalbn(x, sc)), -sc);        /* exact: |x| 2^sc < 2^24 has <= 53 bits */
    return (float)y;                                    /* on the FP32 grid already; >= 2^128 -> inf */
}

/* x rounded down (toward -inf) or up (toward +inf) on the same grid: what "rev" returns. */
static float directed_b(double x, int b_r, int up)
{
    if (isnan(x) || isinf(x) || x == 0.0) return (float)x;
    int sc = grid_scale_exponent(x, b_r);
    double t = scalbn(x, sc);
    double y = scalbn(up ? ceil(t) : floor(t), -sc);
    if (y == 0.0) y = copysign(0.0, x);                 /* keeps the sign of x, like IEEE directed rounding */
    if (fabs(y) >= 0x1p128) {                           /* past the largest finite grid value */
        double top = scalbn(ldexp(1.0, b_r - 8) - 1.0, 127 - (b_r - 9));
        y = (up == (x > 0)) ? copysign(INFINITY, x) : copysign(top, x);
    }
    return (float)y;
}

uint32_t vto_rnd32_bits(double x)
{
    if (isnan(x)) return 0x7FC00000u;
    return f32_bits(rnd32(x));
}

uint32_t vto_thr_from_tau(double tau_ulp)
{
    if (!(tau_ulp >= 0.0 && tau_ulp <= 0.5)) return 0xFFFFFFFFu;
    return (uint32_t)ceil(ldexp(tau_ulp, 29)); /* power-of-two scaling is exact */
}

/* Algorithm "log", steps 1-2: exp = exponent scale of x, then |x - rnd(x)| relative to it.
 * Returned in units of 2^-29 ulp32(x), where every quantity involved is exact in binary64:
 *  - FP32-normal and larger magnitudes: the test does not depend on the binade, so x is
 *    scaled by a power of two into [1,2), where ulp32 = 2^-23 and the unit is 2^-52.
 *  - magnitudes below 2^-126: FP32 spacing is fixed at 2^-149, unit 2^-178. */
/* For b_r < 32 the grid spacing is 2^(32 - b_r) ulp32(x) and the unit is 2^-29 of THAT spacing,
 * so the result is still a real in [0, 2^28] (no longer always an integer). */
double vto_scaled_round_error_b(double x, int b_r)
{
    if (isnan(x) || isinf(x)) return -1.0;
    if (x == 0.0) return 0.0;
    int E = ilogb(x), k = 32 - b_r;
    if (E >= -126) {
        double xs = scalbn(x, -E);                      /* exact, |xs| in [1,2) */
        double d  = fabs(xs - (double)rnd_b(xs, b_r));  /* exact: both are multiples of 2^-52 */
        return ldexp(d, 52 - k);
    } else {
        double d = fabs(x - (double)rnd_b(x, b_r));     /* exact: |d| <= 2^(-150+k) on x's own grid */
        return ldexp(d, 178 - k);
    }
}

double vto_scaled_round_error(double x) { return vto_scaled_round_error_b(x, 32); }

uint32_t vto_boundary_distance_b(double x, int b_r)
{
    double q = vto_scaled_round_error_b(x, b_r);
    if (q < 0.0) return 1u << 28;
    return (uint32_t)(TWO28 - ceil(q)); /* floor(2^28 - q) without rounding the subtraction */
}

uint32_t vto_boundary_distance(double x) { return vto_boundary_distance_b(x, 32); }

uint32_t vto_rnd_b_bits(double x, int b_r)
{
    if (isnan(x)) return 0x7FC00000u;
    return f32_bits(rnd_b(x, b_r));
}

/* Algorithm "log": three-way decision.  exp*tau of the paper equals
 * (0.5 - thr 2^-29) ulp32(x); in the scaled unit that is 2^28 - thr. */
int vto_ternary_code(double x, uint32_t thr) { return vto_ternary_code_b(x, thr, 32); }

int vto_ternary_code_b(double x, uint32_t thr, int b_r)
{
    double q = vto_scaled_round_error_b(x, b_r);
    if (q < 0.0) return 1;                              /* NaN, +-Inf: ignore */
    double y = (double)rnd_b(x, b_r);                   /* may be +-Inf on overflow */
    if (q > TWO28 - (double)thr && x < y) return 2;     /* far from rnd(x), rounded up */
    if (q > TWO28 - (double)thr && x > y) return 0;     /* far from rnd(x), rounded down */
    return 1;
}

int vto_round_log(const double *x, uint64_t n, double tau_ulp, float *y,
                  uint32_t *idx, uint32_t *dir, uint64_t cap, uint64_t *count)
{
    return vto_round_log_b(x, n, tau_ulp, 32, y, idx, dir, cap, count);
}

int vto_round_log_b(const double *x, uint64_t n, double tau_ulp, int b_r, float *y,
                    uint32_t *idx, uint32_t *dir, uint64_t cap, uint64_t *count)
{
    uint32_t thr = vto_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || n >= (1ull << 32) || !count || !valid_br(b_r)) return VTO_ERR_INVALID_ARG;
    if (n && (!x || !y)) return VTO_ERR_INVALID_ARG;
    if (cap && (!idx || !dir)) return VTO_ERR_INVALID_ARG;
    for (uint64_t w = 0; w < (cap + 31) / 32; ++w) dir[w] = 0;
    uint64_t c = 0;
    for (uint64_t i = 0; i < n; ++i) {
        int code = vto_ternary_code_b(x[i], thr, b_r);  /* log(output, ...) first ... */
        y[i] = f32_from(vto_rnd_b_bits(x[i], b_r));     /* ... then output = rnd(output) */
        if (code != 1) {
            if (c < cap) {
                idx[c] = (uint32_t)i;
                if (code == 2) dir[c >> 5] |= 1u << (c & 31);
            }
            ++c;
        }
    }
    *count = c;
    return VTO_OK;
}

/* Primitive "rev" as the paper words it: round to nearest, then, if the trainer went the
 * other way, take the neighbouring FP32 value on the trainer's side of x. */
static float rev(double x, int code, int b_r)
{
    if (isnan(x)) return f32_from(0x7FC00000u);
    float y = rnd_b(x, b_r);
    if (b_r == 32) {
        if (code == 0 && x < (double)y) return nextafterf(y, -INFINITY); /* float below x */
        if (code == 2 && x > (double)y) return nextafterf(y, INFINITY);  /* float above x */
        return y;
    }
    if (code == 0 && x < (double)y) return directed_b(x, b_r, 0);    /* grid point below x */
    if (code == 2 && x > (double)y) return directed_b(x, b_r, 1);    /* grid point above x */
    return y;
}

int vto_round_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                     uint64_t count, float *y)
{
    return vto_round_replay_b(x, n, idx, dir, count, 32, y);
}

int vto_round_replay_b(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                       uint64_t count, int b_r, float *y)
{
    if (n >= (1ull << 32) || !valid_br(b_r)) return VTO_ERR_INVALID_ARG;
    if (n && (!x || !y)) return VTO_ERR_INVALID_ARG;
    if (count && (!idx || !dir)) return VTO_ERR_INVALID_ARG;
    uint64_t p = 0;
    for (uint64_t i = 0; i < n; ++i) {
        int code = 1;                                    /* c = read(F) for element i */
        while (p < count && idx[p] < i) ++p;             /* tolerate stray entries */
        if (p < count && idx[p] == i) {
            code = ((dir[p >> 5] >> (p & 31)) & 1u) ? 2 : 0;
            ++p;
        }
        y[i] = rev(x[i], code, b_r);
    }
    return VTO_OK;
}

uint8_t vto_ternary_pack5(const uint8_t codes[5])
{
    unsigned v = 0, w = 1;
    for (int j = 0; j < 5; ++j) { v += codes[j] * w; w *= 3; }
    return (uint8_t)v;
}

void vto_ternary_unpack5(uint8_t byte, uint8_t codes[5])
{
    unsigned v = byte;
    for (int j = 0; j < 5; ++j) { codes[j] = (uint8_t)(v % 3); v /= 3; }
}

int vto_round_log_dense(const double *x, uint64_t n, double tau_ulp, float *y, uint8_t *tlog,
                        uint64_t *n_logged)
{
    return vto_round_log_dense_b(x, n, tau_ulp, 32, y, tlog, n_logged);
}

int vto_round_log_dense_b(const double *x, uint64_t n, double tau_ulp, int b_r, float *y, uint8_t *tlog,
                          uint64_t *n_logged)
{
    uint32_t thr = vto_thr_from_tau(tau_ulp);
    if (thr == 0xFFFFFFFFu || !valid_br(b_r) || (n && (!x || !y || !tlog))) return VTO_ERR_INVALID_ARG;
    uint64_t logged = 0;
    for (uint64_t k = 0; k * 5 < n; ++k) {
        uint8_t codes[5];
        for (int j = 0; j < 5; ++j) {
            uint64_t i = k * 5 + (uint64_t)j;
            codes[j] = 1;                                    /* past the end: ignore */
            if (i < n) {
                codes[j] = (uint8_t)vto_ternary_code_b(x[i], thr, b_r);
                y[i] = f32_from(vto_rnd_b_bits(x[i], b_r));
                if (codes[j] != 1) ++logged;
            }
        }
        tlog[k] = vto_ternary_pack5(codes);
    }
    if (n_logged) *n_logged = logged;
    return VTO_OK;
}

int vto_round_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, float *y)
{
    return vto_round_replay_dense_b(x, n, tlog, 32, y);
}

int vto_round_replay_dense_b(const double *x, uint64_t n, const uint8_t *tlog, int b_r, float *y)
{
    if (!valid_br(b_r) || (n && (!x || !y || !tlog))) return VTO_ERR_INVALID_ARG;
    for (uint64_t i = 0; i < n; ++i) {
        uint8_t codes[5];
        vto_ternary_unpack5(tlog[i / 5], codes);             /* c = read(F) for element i */
        y[i] = rev(x[i], codes[i % 5], b_r);
    }
    return VTO_OK;
}

int vto_gemm_f64(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                 const double *A, int64_t lda, const double *B, int64_t ldb,
                 const double *bias, double *C, int64_t ldc, int order)
{
    if (M < 0 || N < 0 || K < 0 || order < 0 || order > 2) return VTO_ERR_INVALID_ARG;
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double c;
            if (order == 2) {
                long double acc = 0.0L;
                for (int64_t k = 0; k < K; ++k) {
                    double a = transA ? A[k * lda + i] : A[i * lda + k];
                    double b = transB ? B[j * ldb + k] : B[k * ldb + j];
                    acc += (long double)a * (long double)b;
                }
                long double r = (long double)alpha * acc;
                if (bias) r += (long double)bias[j];
                c = (double)r;
            } else {
                double acc = 0.0;
                for (int64_t s = 0; s < K; ++s) {
                    int64_t k = order == 0 ? s : K - 1 - s;
                    double a = transA ? A[k * lda + i] : A[i * lda + k];
                    double b = transB ? B[j * ldb + k] : B[k * ldb + j];
                    double p = a * b;
                    acc = acc + p;
                }
                c = alpha * acc;
                if (bias) c = c + bias[j];
            }
            C[i * ldc + j] = c;
        }
    }
    return VTO_OK;
}

int vto_conv2d_out_size(const vto_conv2d *d, int64_t *Ho, int64_t *Wo)
{
    if (!d || d->N < 0 || d->H < 0 || d->W < 0 || d->C < 0 || d->KH < 1 || d->KW < 1 || d->stride_h < 1 ||
        d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0 || d->dil_h < 1 || d->dil_w < 1)
        return VTO_ERR_INVALID_ARG;
    int64_t eh = d->H + 2 * d->pad_h - d->dil_h * (d->KH - 1) - 1;
    int64_t ew = d->W + 2 * d->pad_w - d->dil_w * (d->KW - 1) - 1;
    *Ho = eh < 0 ? 0 : eh / d->stride_h + 1;
    *Wo = ew < 0 ? 0 : ew / d->stride_w + 1;
    return VTO_OK;
}

/* X[n,h,w,ci] with zero padding outside the image */
static double conv_x(const vto_conv2d *d, const double *X, int64_t n, int64_t h, int64_t w, int64_t ci)
{
    if (h < 0 || h >= d->H || w < 0 || w >= d->W) return 0.0;
    return X[((n * d->H + h) * d->W + w) * d->C + ci];
}

int vto_conv2d_fwd_f64(const vto_conv2d *d, int64_t Cout, const double *X, const double *Wt,
                       const double *bias, double *Y, int order)
{
    int64_t Ho, Wo;
    if (vto_conv2d_out_size(d, &Ho, &Wo) != VTO_OK || Cout < 0 || order < 0 || order > 2) return VTO_ERR_INVALID_ARG;
    const int64_t taps = d->KH * d->KW * d->C;
    for (int64_t n = 0; n < d->N; ++n)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t co = 0; co < Cout; ++co) {
                    double acc = 0.0;
                    long double accl = 0.0L;
                    for (int64_t s = 0; s < taps; ++s) {
                        int64_t t = order == 1 ? taps - 1 - s : s;
                        int64_t ci = t % d->C, kw = (t / d->C) % d->KW, kh = t / (d->C * d->KW);
                        double x = conv_x(d, X, n, ho * d->stride_h - d->pad_h + kh * d->dil_h,
                                          wo * d->stride_w - d->pad_w + kw * d->dil_w, ci);
                        double w = Wt[((kh * d->KW + kw) * d->C + ci) * Cout + co];
                        if (order == 2) accl += (long double)x * (long double)w;
                        else { double p = x * w; acc = acc + p; }
                    }
                    double y;
                    if (order == 2) { if (bias) accl += (long double)bias[co]; y = (double)accl; }
                    else { y = acc; if (bias) y = y + bias[co]; }
                    Y[((n * Ho + ho) * Wo + wo) * Cout + co] = y;
                }
    return VTO_OK;
}

int vto_conv2d_wgrad_f64(const vto_conv2d *d, int64_t Cout, const double *X, const double *dY,
                         double *dW, int order)
{
    int64_t Ho, Wo;
    if (vto_conv2d_out_size(d, &Ho, &Wo) != VTO_OK || Cout < 0 || order < 0 || order > 2) return VTO_ERR_INVALID_ARG;
    const int64_t pos = d->N * Ho * Wo;
    for (int64_t kh = 0; kh < d->KH; ++kh)
        for (int64_t kw = 0; kw < d->KW; ++kw)
            for (int64_t ci = 0; ci < d->C; ++ci)
                for (int64_t co = 0; co < Cout; ++co) {
                    double acc = 0.0;
                    long double accl = 0.0L;
                    for (int64_t s = 0; s < pos; ++s) {
                        int64_t m = order == 1 ? pos - 1 - s : s;
                        int64_t wo = m % Wo, ho = (m / Wo) % Ho, n = m / (Wo * Ho);
                        double x = conv_x(d, X, n, ho * d->stride_h - d->pad_h + kh * d->dil_h,
                                          wo * d->stride_w - d->pad_w + kw * d->dil_w, ci);
                        double g = dY[m * Cout + co];
                        if (order == 2) accl += (long double)x * (long double)g;
                        else { double p = x * g; acc = acc + p; }
                    }
                    dW[((kh * d->KW + kw) * d->C + ci) * Cout + co] = order == 2 ? (double)accl : acc;
                }
    return VTO_OK;
}

/* Gradient of the forward map with respect to its input (the backward pass of a convolution
 * layer, which the method also computes in FP64 and rounds): dX[n,h,w,ci] is the sum over all
 * (kh, kw, co) of dY[n,ho,wo,co] * W[kh,kw,ci,co] for the output positions whose tap (kh, kw)
 * reads X[n,h,w,.], that is ho * stride - pad + kh * dil = h (likewise in w).  Terms are added in
 * ascending (order 0) or descending (order 1) (kh, kw, co); order 2 accumulates in long double. */
int vto_conv2d_dgrad_f64(const vto_conv2d *d, int64_t Cout, const double *dY, const double *Wt,
                         double *dX, int order)
{
    int64_t Ho, Wo;
    if (vto_conv2d_out_size(d, &Ho, &Wo) != VTO_OK || Cout < 0 || order < 0 || order > 2) return VTO_ERR_INVALID_ARG;
    const int64_t terms = d->KH * d->KW * Cout;
    for (int64_t n = 0; n < d->N; ++n)
        for (int64_t h = 0; h < d->H; ++h)
            for (int64_t w = 0; w < d->W; ++w)
                for (int64_t ci = 0; ci < d->C; ++ci) {
                    double acc = 0.0;
                    long double accl = 0.0L;
                    for (int64_t s = 0; s < terms; ++s) {
                        int64_t t = order == 1 ? terms - 1 - s : s;
                        int64_t co = t % Cout, kw = (t / Cout) % d->KW, kh = t / (Cout * d->KW);
                        int64_t hs = h + d->pad_h - kh * d->dil_h, ws = w + d->pad_w - kw * d->dil_w;
                        double g = 0.0;
                        if (hs >= 0 && ws >= 0 && hs % d->stride_h == 0 && ws % d->stride_w == 0 &&
                            hs / d->stride_h < Ho && ws / d->stride_w < Wo)
                            g = dY[((n * Ho + hs / d->stride_h) * Wo + ws / d->stride_w) * Cout + co];
                        double wv = Wt[((kh * d->KW + kw) * d->C + ci) * Cout + co];
                        if (order == 2) accl += (long double)g * (long double)wv;
                        else { double p = g * wv; acc = acc + p; }
                    }
                    dX[((n * d->H + h) * d->W + w) * d->C + ci] = order == 2 ? (double)accl : acc;
                }
    return VTO_OK;
}

int vto_elementwise_f64(int op, const double *a, const double *b, uint64_t n, double *y, int exact)
{
    if (op < VTO_EW_ADD || op > VTO_EW_GELU_ERF || (n && (!a || !y)) || (op == VTO_EW_ADD && n && !b))
        return VTO_ERR_INVALID_ARG;
    for (uint64_t i = 0; i < n; ++i) {
        double x = a[i];
        if (op == VTO_EW_ADD) {
            y[i] = exact ? (double)((long double)x + (long double)b[i]) : x + b[i];
        } else if (op == VTO_EW_RELU) {
            y[i] = isnan(x) ? x : (x > 0.0 ? x : 0.0);
        } else if (op == VTO_EW_GELU_TANH) {
            if (exact) {
                long double t = (long double)x;
                long double u = sqrtl(2.0L / 3.14159265358979323846264338327950288L) * (t + 0.044715L * t * t * t);
                y[i] = (double)(0.5L * t * (1.0L + tanhl(u)));
            } else {
                double x3 = x * x * x;
                double u = 0.7978845608028654 * (x + 0.044715 * x3);      /* sqrt(2/pi) */
                y[i] = 0.5 * x * (1.0 + tanh(u));
            }
        } else {
            if (exact) {
                long double t = (long double)x;
                y[i] = (double)(0.5L * t * (1.0L + erfl(t / sqrtl(2.0L))));
            } else {
                y[i] = 0.5 * x * (1.0 + erf(x * 0.7071067811865476));     /* 1/sqrt 2 */
            }
        }
    }
    return VTO_OK;
}

int vto_layernorm_f64(const double *x, int64_t rows, int64_t cols, const double *gamma, const double *beta,
                      double eps, double *y, int order)
{
    if (rows < 0 || cols < 0 || order < 0 || order > 2 || (rows > 0 && cols > 0 && (!x || !y))) return VTO_ERR_INVALID_ARG;
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * cols;
        double *yr = y + r * cols;
        if (order == 2) {
            long double s = 0.0L, q = 0.0L;
            for (int64_t c = 0; c < cols; ++c) s += (long double)xr[c];
            long double mean = s / (long double)cols;
            for (int64_t c = 0; c < cols; ++c) { long double d = (long double)xr[c] - mean; q += d * d; }
            long double rstd = 1.0L / sqrtl(q / (long double)cols + (long double)eps);
            for (int64_t c = 0; c < cols; ++c) {
                long double v = ((long double)xr[c] - mean) * rstd;
                if (gamma) v *= (long double)gamma[c];
                if (beta) v += (long double)beta[c];
                yr[c] = (double)v;
            }
        } else {
            double s = 0.0, q = 0.0;
            for (int64_t t = 0; t < cols; ++t) s = s + xr[order ? cols - 1 - t : t];
            double mean = s / (double)cols;
            for (int64_t t = 0; t < cols; ++t) { double d = xr[order ? cols - 1 - t : t] - mean; q = q + d * d; }
            double rstd = 1.0 / sqrt(q / (double)cols + eps);
            for (int64_t c = 0; c < cols; ++c) {
                double v = (xr[c] - mean) * rstd;
                if (gamma) v = v * gamma[c];
                if (beta) v = v + beta[c];
                yr[c] = v;
            }
        }
    }
    return VTO_OK;
}

int vto_batchnorm_f64(const double *x, int64_t rows, int64_t cols, const double *gamma, const double *beta,
                      double eps, int relu, double *y, int order)
{
    if (rows < 0 || cols < 0 || order < 0 || order > 2 || (rows > 0 && cols > 0 && (!x || !y))) return VTO_ERR_INVALID_ARG;
    for (int64_t c = 0; c < cols; ++c) {
        long double meanl = 0.0L, rstdl = 0.0L;
        double mean = 0.0, rstd = 0.0;
        if (order == 2) {
            long double s = 0.0L, q = 0.0L;
            for (int64_t r = 0; r < rows; ++r) s += (long double)x[r * cols + c];
            meanl = s / (long double)rows;
            for (int64_t r = 0; r < rows; ++r) { long double d = (long double)x[r * cols + c] - meanl; q += d * d; }
            rstdl = 1.0L / sqrtl(q / (long double)rows + (long double)eps);
        } else {
            double s = 0.0, q = 0.0;
            for (int64_t t = 0; t < rows; ++t) s = s + x[(order ? rows - 1 - t : t) * cols + c];
            mean = s / (double)rows;
            for (int64_t t = 0; t < rows; ++t) { double d = x[(order ? rows - 1 - t : t) * cols + c] - mean; q = q + d * d; }
            rstd = 1.0 / sqrt(q / (double)rows + eps);
        }
        for (int64_t r = 0; r < rows; ++r) {
            double v;
            if (order == 2) {
                long double w = ((long double)x[r * cols + c] - meanl) * rstdl;
                if (gamma) w *= (long double)gamma[c];
                if (beta) w += (long double)beta[c];
                v = (double)w;
            } else {
                v = (x[r * cols + c] - mean) * rstd;
                if (gamma) v = v * gamma[c];
                if (beta) v = v + beta[c];
            }
            if (relu) v = isnan(v) ? v : (v > 0.0 ? v : 0.0);
            y[r * cols + c] = v;
        }
    }
    return VTO_OK;
}

int vto_softmax_f64(const double *x, int64_t rows, int64_t cols, double scale, int64_t causal_period,
                    double *y, int order)
{
    if (rows < 0 || cols < 0 || causal_period < 0 || order < 0 || order > 2 || (rows > 0 && cols > 0 && (!x || !y)))
        return VTO_ERR_INVALID_ARG;
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * cols;
        double *yr = y + r * cols;
        int64_t seen = causal_period > 0 ? r % causal_period + 1 : cols;   /* columns 0 .. seen-1 are visible */
        if (seen > cols) seen = cols;
        double m = -INFINITY;
        for (int64_t c = 0; c < seen; ++c) { double z = scale * xr[c]; if (z > m) m = z; }
        if (order == 2) {
            long double s = 0.0L;
            for (int64_t c = 0; c < seen; ++c) s += expl((long double)scale * (long double)xr[c] - (long double)m);
            for (int64_t c = 0; c < cols; ++c)
                yr[c] = c < seen ? (double)(expl((long double)scale * (long double)xr[c] - (long double)m) / s) : 0.0;
        } else {
            double s = 0.0;
            for (int64_t t = 0; t < seen; ++t) { int64_t c = order ? seen - 1 - t : t; s = s + exp(scale * xr[c] - m); }
            double inv = 1.0 / s;
            for (int64_t c = 0; c < cols; ++c) yr[c] = c < seen ? exp(scale * xr[c] - m) * inv : 0.0;
        }
    }
    return VTO_OK;
}

/* Monotone integer image of a binary64 pattern: sign-magnitude -> two's complement. */
static int64_t ord64(double y)
{
    uint64_t b = f64_bits(y);
    uint64_t mag = b & 0x7FFFFFFFFFFFFFFFull;
    return (b >> 63) ? -(int64_t)mag : (int64_t)mag;
}

int vto_threshold_stats(const double *y1, const double *y2, uint64_t n, uint64_t out[68])
{
    return vto_threshold_stats_b(y1, y2, n, 32, out);
}

int vto_threshold_stats_b(const double *y1, const double *y2, uint64_t n, int b_r, uint64_t out[68])
{
    if (!out || !valid_br(b_r) || (n && (!y1 || !y2))) return VTO_ERR_INVALID_ARG;
    for (int b = 0; b < 68; ++b) out[b] = 0;
    for (uint64_t i = 0; i < n; ++i) {
        int64_t o1 = ord64(y1[i]), o2 = ord64(y2[i]);
        uint64_t diff = o1 > o2 ? (uint64_t)o1 - (uint64_t)o2 : (uint64_t)o2 - (uint64_t)o1;
        int bin = 0;
        for (uint64_t d = diff; d; d >>= 1) ++bin;      /* 0, else 1 + floor(log2 diff) */
        out[3 + bin] += 1;
        if (diff > out[2]) out[2] = diff;
        if (vto_rnd_b_bits(y1[i], b_r) != vto_rnd_b_bits(y2[i], b_r)) {   /* rnd(y1) != rnd(y2) */
            uint32_t d1 = vto_boundary_distance_b(y1[i], b_r);
            uint32_t d2 = vto_boundary_distance_b(y2[i], b_r);
            uint64_t need = 1 + (uint64_t)(d1 > d2 ? d1 : d2);
            out[0] += 1;
            if (need > out[1]) out[1] = need;
        }
    }
    return VTO_OK;
}
