/*
 * vt_oracle.h -- plain CPU oracle for the verifiable-training round/log/replay path.
 *
 * TEST INFRASTRUCTURE ONLY.  This code is the slow, scalar, obviously-correct statement of
 * what the method computes, written from the paper (Method section: primitives rnd, log,
 * rev, threshold; Appendix algorithms "log", "audit", "threshold").  It shares no code with
 * the HIP library and must never be called from the product path; only the tests, the smoke
 * check and the bench's cpu_baseline leg use it.
 *
 * Conventions (the paper's quantities restated exactly):
 *   ulp32(x)  spacing of FP32 numbers at x: 2^(max(E,-126)-23), E = floor(log2|x|).
 *   tau_ulp   threshold measured from the rounding boundary (FP32 midpoint) in units of
 *             ulp32(x).  The paper's tau (distance from the rounded value, written c*2^-23)
 *             maps to tau_ulp = 0.5 - c.
 *   thr       integer threshold ceil(tau_ulp * 2^29) in [0, 2^28]; one unit is the FP64
 *             spacing inside an FP32-normal binade.
 *   logged    |x - rnd(x)| > (0.5 - thr*2^-29) * ulp32(x)          (Algorithm "log")
 *   dir       1 when rnd(x) > x (rounded toward +inf, the paper's code 2), else 0 (code 0)
 *   log       ascending element indices of logged elements + one direction bit each,
 *             bit (p & 31) of word dir[p >> 5] for entry p.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py against exact
 * rational arithmetic, library routines, closed forms and brute force -- except the NaN
 * payload convention (canonical 0x7FC00000), which is a convention of this build
 * ("parity unpinned").
 */
#ifndef VT_ORACLE_H
#define VT_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VTO_OK 0
#define VTO_ERR_INVALID_ARG 1

/* rnd_32: IEEE binary64 -> binary32 conversion, round to nearest, ties to even.
 * Returns the FP32 bit pattern; NaN inputs give 0x7FC00000. (Method, primitive 1.) */
uint32_t vto_rnd32_bits(double x);

/* ceil(tau_ulp * 2^29); returns 0xFFFFFFFF when tau_ulp is outside [0, 0.5] or NaN. */
uint32_t vto_thr_from_tau(double tau_ulp);

/* Scaled distance to the rounded value, q = |x - rnd(x)| / (2^-29 ulp32(x)), a real in
 * [0, 2^28].  For |x| >= 2^-126 the test is exponent-invariant, so x is first scaled into
 * [1,2); this extends the FP32 grid past FLT_MAX for values that overflow to infinity.
 * Returns -1 for NaN and +-Inf (never logged). (Algorithm "log", first two steps.) */
double vto_scaled_round_error(double x);

/* floor(2^28 - q): the boundary distance in threshold units; 2^28 for NaN/Inf. */
uint32_t vto_boundary_distance(double x);

/* Paper's ternary code for one element: 2 = logged, rounded up; 0 = logged, rounded down;
 * 1 = ignore. (Algorithm "log".) */
int vto_ternary_code(double x, uint32_t thr);

/* Trainer side: y[i] = rnd_32(x[i]); logged elements appended to idx/dir in ascending i.
 * *count receives the number of logged elements even when it exceeds cap (then only the
 * first cap entries are stored).  n must be < 2^32. */
int vto_round_log(const double *x, uint64_t n, double tau_ulp, float *y,
                  uint32_t *idx, uint32_t *dir, uint64_t cap, uint64_t *count);

/* Auditor side (primitive "rev", Algorithm "audit"): unlogged i -> rnd_32(x[i]); logged i
 * -> rnd_32(x[i]) stepped one FP32 value toward the logged direction when it lies on the
 * other side of x[i]. */
int vto_round_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                     uint64_t count, float *y);

/* The log as the paper stores it (Method, "Reducing storage cost"): one ternary entry per
 * output -- 2 rounded up, 0 rounded down, 1 ignore -- in element order, five entries per byte by
 * radix-3 to radix-2 conversion (3^5 = 243 <= 256, 1.6 bits per entry).  Reading taken here:
 * byte k holds elements 5k .. 5k+4, element 5k+j as the digit of weight 3^j; positions past the
 * end of the tensor hold 1.  The log of n outputs is ceil(n/5) bytes. */
uint8_t vto_ternary_pack5(const uint8_t codes[5]);
void vto_ternary_unpack5(uint8_t byte, uint8_t codes[5]);   /* digit j = (byte / 3^j) % 3 for any byte */

/* Trainer side with the packed ternary log: y[i] = rnd_32(x[i]), tlog = ceil(n/5) bytes;
 * *n_logged (optional) receives the number of entries that are not 1. */
int vto_round_log_dense(const double *x, uint64_t n, double tau_ulp, float *y, uint8_t *tlog,
                        uint64_t *n_logged);

/* Auditor side: entry i of the packed log applied to x[i] with "rev". */
int vto_round_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, float *y);

/* Scalar FP64 GEMM, C[i,j] = alpha * sum_k opA(i,k) opB(k,j) (+ bias[j]), no contraction.
 * order 0: k ascending; 1: k descending; 2: long double accumulation ("truth").
 * Row-major storage; transX != 0 means the operand is stored transposed. */
int vto_gemm_f64(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                 const double *A, int64_t lda, const double *B, int64_t ldb,
                 const double *bias, double *C, int64_t ldc, int order);

/* A 2-D convolution layer, the other "intermediate computation" the method rounds after
 * (Method, "rounding after intermediate computations, e.g. a convolution"; Experiments,
 * ResNet-50; Algorithm "train" rounds forward outputs and gradients alike).  Cross-correlation
 * with zero padding, as deep-learning layers define it; channels-last storage:
 *   X [N][H][W][C],  Wt [KH][KW][C][Cout],  Y, dY [N][Ho][Wo][Cout],
 *   Ho = (H + 2 pad_h - dil_h (KH-1) - 1) / stride_h + 1  (floor), Wo alike. */
typedef struct vto_conv2d {
    int64_t N, H, W, C, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} vto_conv2d;

int vto_conv2d_out_size(const vto_conv2d *d, int64_t *Ho, int64_t *Wo);

/* Y[n,ho,wo,co] = sum_{kh,kw,ci} X[n, ho s - p + kh dil, wo s - p + kw dil, ci] Wt[kh,kw,ci,co]
 * (+ bias[co]); taps that fall into the padding contribute nothing.
 * order 0: taps in ascending (kh,kw,ci); 1: descending; 2: long double accumulation. */
int vto_conv2d_fwd_f64(const vto_conv2d *d, int64_t Cout, const double *X, const double *Wt,
                       const double *bias, double *Y, int order);

/* Gradient of sum(Y * dY) with respect to the weights:
 * dW[kh,kw,ci,co] = sum_{n,ho,wo} X[n, ho s - p + kh dil, wo s - p + kw dil, ci] dY[n,ho,wo,co].
 * order 0: output positions in ascending (n,ho,wo); 1: descending; 2: long double. */
int vto_conv2d_wgrad_f64(const vto_conv2d *d, int64_t Cout, const double *X, const double *dY,
                         double *dW, int order);

/* Gradient of sum(Y * dY) with respect to the input:
 * dX[n,h,w,ci] = sum_{kh,kw,co} dY[n,ho,wo,co] Wt[kh,kw,ci,co] over the (ho, wo) with
 * ho s - p + kh dil = h and wo s - p + kw dil = w (none when the difference is not a multiple of
 * the stride or falls outside the output).
 * order 0: terms in ascending (kh,kw,co); 1: descending; 2: long double. */
int vto_conv2d_dgrad_f64(const vto_conv2d *d, int64_t Cout, const double *dY, const double *Wt,
                         double *dX, int order);

/* The same primitives with a rounding amount b_r < 32 (Method, primitives rnd_{b_r}, log, rev;
 * caption of the floating-point figure: the nearest 32-bit float with zeros in the last 32 - b_r
 * mantissa bits).  The grid spacing is 2^(32 - b_r) ulp32(x); tau_ulp and thr are measured in
 * units of THAT spacing (thr = ceil(tau_ulp 2^29) as before), so the threshold search range
 * [0.25, 0.5] x spacing keeps its meaning.  10 <= b_r <= 32; b_r = 32 is the functions above. */
uint32_t vto_rnd_b_bits(double x, int b_r);
double vto_scaled_round_error_b(double x, int b_r);
uint32_t vto_boundary_distance_b(double x, int b_r);
int vto_ternary_code_b(double x, uint32_t thr, int b_r);
int vto_round_log_b(const double *x, uint64_t n, double tau_ulp, int b_r, float *y,
                    uint32_t *idx, uint32_t *dir, uint64_t cap, uint64_t *count);
int vto_round_replay_b(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                       uint64_t count, int b_r, float *y);
int vto_round_log_dense_b(const double *x, uint64_t n, double tau_ulp, int b_r, float *y, uint8_t *tlog,
                          uint64_t *n_logged);
int vto_round_replay_dense_b(const double *x, uint64_t n, const uint8_t *tlog, int b_r, float *y);
int vto_threshold_stats_b(const double *y1, const double *y2, uint64_t n, int b_r, uint64_t out[68]);

/* The other intermediate computations of a network whose outputs the method rounds (Method:
 * "after every intermediate computation"; Table "thresholds" lists layer norm and batch norm next to
 * convolution and linear layers): the element-wise and row-wise layers of a transformer block, by
 * their textbook definitions, in FP64.
 *   VTO_EW_ADD        y = a + b                                   (residual connection)
 *   VTO_EW_RELU       y = x if x > 0, +0 otherwise (NaN stays NaN)
 *   VTO_EW_GELU_TANH  y = x/2 (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3)))
 *   VTO_EW_GELU_ERF   y = x/2 (1 + erf(x / sqrt 2))
 * exact = 0: one binary64 operation per step in the order written; exact = 1: long double. */
#define VTO_EW_ADD 0
#define VTO_EW_RELU 1
#define VTO_EW_GELU_TANH 2
#define VTO_EW_GELU_ERF 3
int vto_elementwise_f64(int op, const double *a, const double *b, uint64_t n, double *y, int exact);

/* Layer normalisation of each row: mean = sum x / cols, var = sum (x - mean)^2 / cols (biased),
 * y = (x - mean) / sqrt(var + eps) * gamma + beta (gamma, beta optional, per column).
 * order 0: sums over ascending columns, 1: descending, 2: long double. */
int vto_layernorm_f64(const double *x, int64_t rows, int64_t cols, const double *gamma, const double *beta,
                      double eps, double *y, int order);

/* Batch normalisation in training mode (Table "thresholds" lists it): per column (channel)
 * mean = sum over rows / rows, var = sum (x - mean)^2 / rows (biased), y = (x - mean) /
 * sqrt(var + eps) * gamma + beta, followed by ReLU when relu != 0.  Rows are the N*H*W positions
 * of a channels-last activation.  order 0: sums over ascending rows, 1: descending, 2: long double. */
int vto_batchnorm_f64(const double *x, int64_t rows, int64_t cols, const double *gamma, const double *beta,
                      double eps, int relu, double *y, int order);

/* Softmax of each row of z = scale * x: y_c = exp(z_c - max z) / sum exp(z - max z).  With
 * causal_period T > 0, row r sees only columns c <= r mod T (attention over a sequence of T tokens,
 * rows stacked head after head); the other outputs are 0.  order as above. */
int vto_softmax_f64(const double *x, int64_t rows, int64_t cols, double scale, int64_t causal_period,
                    double *y, int order);

/* Threshold statistics over two results of the same operation (Algorithm "threshold",
 * collection loop): out[0] = number of elements whose FP32 roundings differ (bit patterns),
 * out[1] = 1 + max over those of max(D(y1), D(y2)) (0 when there are none),
 * out[2] = max |ord(y1) - ord(y2)| in FP64 steps, out[3+b] = histogram: b = 0 for equal,
 * else 1 + floor(log2(steps)). */
int vto_threshold_stats(const double *y1, const double *y2, uint64_t n, uint64_t out[68]);

#ifdef __cplusplus
}
#endif
#endif
