/*
 * vt.h -- C ABI of the verifiable-training hot path on MI355X (gfx950).
 *
 * The library implements the per-layer hook of "Optimistic Verifiable Training by Controlling
 * Hardware Nondeterminism": a layer is computed in FP64, every output is rounded to FP32, and
 * the rounding direction of every output that lies close to an FP32 rounding boundary is
 * recorded in a log; an auditor who recomputed the layer with a different accumulation order
 * replays that log and ends with bit-identical FP32 values (paper: Method section, primitives
 * rnd / log / rev / threshold; Appendix algorithms "train", "audit", "log", "threshold").
 *
 * General conventions
 *   - Every pointer named in a "device" role is DEVICE memory owned by the caller (for example
 *     a PyTorch tensor's data_ptr()).  The library never allocates, frees or retains device
 *     memory; scratch space is passed in as `ws` and sized with vt_workspace_bytes().
 *   - `hip_stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work on it and
 *     return without synchronising; outputs are valid once the stream has been synchronised.
 *   - The return value is a host-side status (VT_OK or a VT_ERR_* code); argument errors are
 *     detected before anything is enqueued.  vt_strerror() names a code.
 *   - Same inputs (and same `variant`) give bit-identical outputs on every run: no kernel uses
 *     floating-point atomics or a timing-dependent summation order.
 *   - Calls may be recorded by stream capture into a HIP graph and replayed: they allocate nothing,
 *     never synchronise, and clear their counters with kernels (no memset nodes).  Host-side
 *     arguments (sizes, thresholds, a replay's entry count) are fixed at capture.
 *
 * Threshold
 *   `tau_ulp` is the logging threshold measured from the rounding boundary (the midpoint
 *   between two neighbouring FP32 values) in units of ulp32(x), the FP32 spacing at x.  The
 *   paper states its threshold tau as a distance from the *rounded value*, tau = c * 2^-23
 *   with c in [0.25, 0.5] (Method, "Reducing storage cost"; Algorithm "log" logs when
 *   |x - rnd(x)| > exp * tau); the two describe the same set with tau_ulp = 0.5 - c.
 *   The library quantises once on the host: thr = ceil(tau_ulp * 2^29), so one unit of thr is
 *   one FP64 step inside an FP32-normal binade, and an element is logged iff its boundary
 *   distance D(x) < thr.  tau_ulp must lie in [0, 0.5].  thr = 1 logs exact ties only.
 *
 * The log (one segment per call; the caller sequences segments, Algorithm "audit" reads them
 * in the same order)
 *   idx[p]   linear index of the p-th logged output, ascending in p
 *   dir      one bit per entry: bit (p & 31) of word dir[p >> 5]; 1 = rnd(x) > x (the paper's
 *            code 2, "up", toward +infinity also for negative x), 0 = rnd(x) < x (code 0)
 *   count    number of logged outputs.  If it exceeds `cap`, only the first `cap` entries (in
 *            canonical order) are stored; all other outputs of the call are still complete,
 *            and the caller may re-run with a larger log.
 *            One value is not a count: VT_COUNT_ABANDONED (all ones).  The single-pass kernel behind
 *            vt_round_log, vt_layer_f64_round_log and the split-K / strided input-gradient routes
 *            orders its tiles' entries through bounded waits inside one launch; if a wait runs out
 *            (tens of seconds without progress: not seen in practice, it would take the GPU
 *            withholding part of the launch that long) the kernel drains instead of hanging and
 *            reports this value.  The FP32 outputs are then complete and correct, idx / dir are not
 *            a valid log, and a larger `cap` does not help: run the call again.
 *   Unlogged outputs are the paper's code 1 ("ignore").
 *
 * The same decisions in the paper's own storage format (Method, "Reducing storage cost"): when
 * `dense` is not NULL the call writes one ternary entry per output instead -- 2 rounded up,
 * 0 rounded down, 1 ignore -- in output order, five entries per byte by radix-3 to radix-2
 * conversion: byte k holds outputs 5k .. 5k+4, output 5k+j with weight 3^j, and the tail of the
 * last byte holds 1.  The buffer is ceil(total / 5) bytes, 4-byte aligned; `cap` must then be 0
 * (idx and dir are not used) and `count` still receives the number of entries that are not 1.
 * 1.6 bits per output whatever the density: smaller than the index list once more than about
 * 5 % of the outputs are logged.
 *
 * Rounding amount (Method, primitives rnd_{b_r}, log, rev; caption of the floating-point figure):
 * `b_r` = 32 (or 0) rounds to FP32.  10 <= b_r < 32 rounds to the nearest 32-bit float whose last
 * 32 - b_r mantissa bits are zero (b_r - 9 mantissa bits; 16 is bfloat16's grid); outputs are
 * still stored as FP32.  The grid spacing is then 2^(32 - b_r) ulp32(x), and tau_ulp, thr and
 * the statistics are measured relative to THAT spacing, so [0, 0.5] keeps its meaning.  The
 * auditor passes the same b_r to the *_br replay and statistics calls.
 */
#ifndef VT_H
#define VT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VT_OK 0
#define VT_ERR_INVALID_ARG 1   /* null / negative / misaligned argument, tau_ulp outside [0,0.5], size limit */
#define VT_ERR_WORKSPACE 2     /* ws is NULL or smaller than vt_workspace_bytes() */
#define VT_ERR_HIP 3           /* a HIP call or kernel launch failed */
#define VT_ERR_UNSUPPORTED 4   /* valid request this build has no kernel for */
#define VT_ERR_STATIC_LIMIT 5  /* vt_round_log_static: n beyond VT_ROUND_LOG_STATIC_MAX_N */

/* *count after a call whose ordered-log pass gave up a bounded wait (see "The log" above). */
#define VT_COUNT_ABANDONED UINT64_MAX

/* Operation selector for vt_workspace_bytes(). */
#define VT_OP_ROUND_LOG 0      /* element count n = M * N * batch, K ignored */
#define VT_OP_ROUND_REPLAY 1   /* needs no workspace (returns 0) */
#define VT_OP_GEMM_ROUND_LOG 2
#define VT_OP_THRESHOLD_STATS 3 /* needs no workspace (returns 0) */
#define VT_OP_GEMM_ROUND_LOG_BR 4 /* GEMM / convolution with log->b_r below 32 (rounds in a second pass) */
#define VT_OP_LAYER_ROUND_LOG 5  /* vt_layer_f64_round_log: M = rows, N = cols */
#define VT_OP_SHA256_TREE 6      /* vt_sha256_tree: N = bytes, K = chunk (M, batch ignored) */
#define VT_OP_MERKLE_ROOT 7      /* vt_merkle_root: N = leaves (M, K, batch ignored) */
#define VT_OP_CONV_DGRAD_ROUND_LOG 8     /* vt_conv2d_f64_round_log, VT_CONV_DATA_GRAD: (M, N, K) of its GEMM */
#define VT_OP_CONV_DGRAD_ROUND_LOG_BR 9  /* the same with log->b_r below 32 */

/* Caller-owned log buffers (all four pointers are device pointers). */
typedef struct vt_log {
    uint32_t *idx;    /* [cap]            ascending linear indices of logged outputs      */
    uint32_t *dir;    /* [ceil(cap / 32)] packed direction bits, see above                */
    uint64_t  cap;    /* capacity in entries                                              */
    uint64_t *count;  /* device scalar: number of logged outputs (may exceed cap)         */
    uint8_t  *dense;  /* NULL, or [ceil(total / 5)] packed ternary log (then cap must be 0) */
    int32_t   b_r;    /* rounding amount: 0 or 32 = FP32, else 10 .. 31                    */
} vt_log;

/*
 * Trainer side on a flat FP64 array (Algorithm "train", forward and backward loops: the log
 * step followed by the rounding step on each layer's output, here with b_r = 32;
 * Algorithm "log" for the decision).
 *   x        device, n FP64 values (8-byte aligned)
 *   y        device, n FP32 values: y[i] = rnd_32(x[i]), IEEE round-to-nearest-even; NaN inputs
 *            give the canonical quiet NaN 0x7FC00000; overflow gives +-infinity
 *   log      host struct of device pointers; must not be NULL; log->count must not be NULL;
 *            idx/dir may be NULL only if cap == 0
 *   ws       device scratch of at least vt_workspace_bytes(VT_OP_ROUND_LOG, 1, n, 0, 1) bytes,
 *            256-byte aligned; contents are overwritten
 *   n        0 <= n < 2^32 (indices are 32-bit)
 */
int vt_round_log(const double *x, uint64_t n, double tau_ulp, float *y, const vt_log *log,
                 void *ws, size_t ws_bytes, void *hip_stream);

/*
 * vt_round_log for callers that cannot allocate device memory and have no workspace to pass: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * outputs and errors as vt_round_log, minus `ws`: the kernels' scratch (the status words of the
 * single-pass kernel, or the counters of the packed-log kernel) lives in a device array inside the
 * library, 2 MiB + 16 KiB per GPU, held until the process ends.  The call allocates and frees nothing.
 *   n        at most VT_ROUND_LOG_STATIC_MAX_N (VT_ERR_STATIC_LIMIT above it; nothing is enqueued)
 *   x, y     with the index-list log (log->dense NULL) x must be 16-byte and y 8-byte aligned
 *            (VT_ERR_UNSUPPORTED otherwise: the fallback for other alignments needs n / 4 bytes of
 *            scratch); the packed ternary log takes any 8-byte / 4-byte aligned pair
 *   The GPU that is current at the call must be the one `hip_stream` and the buffers belong to; the
 *   first call on a GPU looks the array's address up once (make that call outside stream capture).
 *   Every call on one GPU shares that GPU's array: calls that may overlap in time there (two streams,
 *   two host threads) race on it and give unspecified logs -- serialise them, or use vt_round_log
 *   with workspaces of the caller's own.  The kernels clear what they use, so calls made one after
 *   the other need nothing in between.
 */
#define VT_ROUND_LOG_STATIC_MAX_N (1ull << 30)
int vt_round_log_static(const double *x, uint64_t n, double tau_ulp, float *y, const vt_log *log,
                        void *hip_stream);

/*
 * Auditor side (primitive "rev"; Algorithm "audit", the read-and-reverse step after each layer).
 *   x            device, the auditor's own n FP64 results
 *   idx, dir     device, the trainer's log segment for this tensor (count entries, idx ascending)
 *   count        host value: entries in the segment
 *   y            device, n FP32 values: unlogged i -> rnd_32(x[i]); logged i -> x[i] rounded toward
 *                the logged direction (the FP32 neighbour of x[i] on the trainer's side), which is
 *                what "rev" produces from rnd_32(x[i]) and one nextafter step.
 *   Entries whose index is >= n are ignored.  If idx is not ascending the result is unspecified
 *   (but every access stays in bounds).  No workspace is used (ws may be NULL).
 */
int vt_round_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                    uint64_t count, float *y, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Auditor side from the packed ternary log (same primitive "rev"; the log is positional, so entry
 * i is read for output i as Algorithm "audit" does).
 *   tlog     device, ceil(n / 5) bytes as written through vt_log.dense, 4-byte aligned.  Bytes
 *            above 242 (never written by the trainer) decode digit by digit, the sixth dropped.
 */
int vt_round_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, float *y, void *hip_stream);

/* The two auditor calls above for a log that was written with rounding amount b_r (10 .. 32). */
int vt_round_replay_br(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                       uint64_t count, int b_r, float *y, void *hip_stream);
int vt_round_replay_dense_br(const double *x, uint64_t n, const uint8_t *tlog, int b_r, float *y, void *hip_stream);

/*
 * The layer itself, fused with the trainer hook (Algorithm "train": the layer evaluated in
 * b_tr = 64, then log and rnd; the Nondeterminism Challenge section names the tiling of
 * GEMMs as the source of divergence this controls).
 *
 *   C64[b,i,j] = alpha * sum_k opA[b,i,k] * opB[b,k,j]  (+ bias[j])        in FP64 (MFMA)
 *   C32[b,i,j] = rnd_32(C64[b,i,j]);  decisions logged with linear index (b*M + i)*N + j.
 *
 *   transA/transB  0: operand stored row-major as op(X) (A: M x K, B: K x N);
 *                  1: stored transposed (A: K x M, B: N x K), still row-major
 *   lda, ldb, ldc  row pitches in elements; strideA/B/C: element offsets between batches
 *                  (strideA or strideB may be 0 to share an operand)
 *   bias           device, N FP64 values added after the alpha scaling, or NULL
 *   C32            device, FP32 output, row pitch ldc >= N; with batch > 1 the matrices must not
 *                  overlap: one after the other (strideC >= (M - 1) * ldc + N) or side by side in
 *                  the columns of one wide matrix (strideC >= N, (batch - 1) * strideC + N <= ldc)
 *   C64_debug      device or NULL: when given, receives the FP64 values before rounding
 *                  (dense, pitch N, batch stride M*N) -- for tests and threshold statistics
 *   variant        accumulation order: 0 = k steps (and split-K slices) in ascending order;
 *                  1 = in descending order.  Different variants give FP64 results that differ
 *                  in their low bits, as two GPU types would.
 *   M*N*batch must be < 2^32.  A, B 8-byte aligned.
 *   ws             at least vt_workspace_bytes(VT_OP_GEMM_ROUND_LOG, M, N, K, batch) bytes.
 *   With log->b_r below 32 the FP64 result goes through memory once and is rounded by the
 *   standalone hook (the fused epilogue uses the hardware's FP32 conversion): C32 must then be
 *   dense (ldc == N, strideC == M*N; VT_ERR_UNSUPPORTED otherwise) and ws is sized with
 *   VT_OP_GEMM_ROUND_LOG_BR.
 */
int vt_gemm_f64_round_log(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                          const double *A, int64_t lda, int64_t strideA,
                          const double *B, int64_t ldb, int64_t strideB,
                          const double *bias, int64_t batch,
                          float *C32, int64_t ldc, int64_t strideC,
                          double *C64_debug, int variant,
                          double tau_ulp, const vt_log *log,
                          void *ws, size_t ws_bytes, void *hip_stream);

/*
 * The same layer for operands that are batched on two levels, as the attention scores of a
 * transformer are: Q and K of head h of sequence b are column slices of one QKV activation
 * [sequence][token][3][head][64], so consecutive heads lie strideA apart and consecutive sequences
 * strideA_outer apart.  Matrix (o, i), o < batch_outer, i < batch_inner, reads
 *   A + o * strideA_outer + i * strideA   and   B + o * strideB_outer + i * strideB;
 * its outputs are batch element b = o * batch_inner + i of C32 / C64_debug / the log, exactly as
 * vt_gemm_f64_round_log numbers them (ws is sized with batch = batch_inner * batch_outer).  One call
 * keeps every compute unit busy where one call per sequence would not.  Everything else as above.
 */
int vt_gemm_f64_round_log_nested(int transA, int transB, int64_t M, int64_t N, int64_t K, double alpha,
                                 const double *A, int64_t lda, int64_t strideA, int64_t strideA_outer,
                                 const double *B, int64_t ldb, int64_t strideB, int64_t strideB_outer,
                                 const double *bias, int64_t batch_inner, int64_t batch_outer,
                                 float *C32, int64_t ldc, int64_t strideC,
                                 double *C64_debug, int variant,
                                 double tau_ulp, const vt_log *log,
                                 void *ws, size_t ws_bytes, void *hip_stream);

/*
 * A convolution layer fused with the trainer hook (the paper's other example of an
 * intermediate computation: Method; Experiments, ResNet-50;
 * Algorithm "train" rounds and logs forward outputs and gradients alike).  The layer is the GEMM
 * above over the im2col matrix of the image, which is never materialised: the kernel forms the
 * addresses while it loads.  Cross-correlation with zero padding, channels last:
 *
 *   VT_CONV_FORWARD      Y[n,ho,wo,co]   = sum_{kh,kw,ci} X[n, ho s - p + kh d, wo s - p + kw d, ci] Wt[kh,kw,ci,co] (+ bias[co])
 *                        B = Wt [KH][KW][C][Cout];  C32 = Y [N][Ho][Wo][Cout]
 *   VT_CONV_WEIGHT_GRAD  dW[kh,kw,ci,co] = sum_{n,ho,wo} X[n, ho s - p + kh d, wo s - p + kw d, ci] dY[n,ho,wo,co]
 *                        B = dY [N][Ho][Wo][Cout];  C32 = dW [KH][KW][C][Cout];  bias must be NULL
 *   VT_CONV_DATA_GRAD    dX[n,h,w,ci]    = sum_{kh,kw,co} dY[n,ho,wo,co] Wt[kh,kw,ci,co] over the output positions
 *                        with ho s - p + kh d = h and wo s - p + kw d = w (the gradient with respect to the
 *                        layer's input).  The argument X is dY [N][Ho][Wo][Cout] (read through the matching
 *                        implicit view, zeros where no output position reads the input position);
 *                        B = Wt [KH][KW][C][Cout];  C32 = dX [N][H][W][C];  bias must be NULL.  The geometry
 *                        `d` is the forward layer's (N, H, W, C describe the layer's input).
 *   Ho = floor((H + 2 pad_h - dil_h (KH - 1) - 1) / stride_h) + 1, Wo alike.
 *
 *   X            device, the image batch [N][H][W][C], dense, 8-byte aligned (16-byte alignment and
 *                an even C let the kernel use 16-byte loads)
 *   C32, C64_debug, variant, tau_ulp, log: as for vt_gemm_f64_round_log; outputs are dense; the
 *                log index of an output is its linear index in C32.  variant 0 accumulates taps
 *                (forward) or output positions (weight gradient) in ascending order, 1 descending.
 *   ws           at least vt_workspace_bytes(VT_OP_GEMM_ROUND_LOG, M, N, K, 1) bytes for the
 *                (M, N, K) that vt_conv2d_gemm_shape reports; for VT_CONV_DATA_GRAD
 *                vt_workspace_bytes(VT_OP_CONV_DGRAD_ROUND_LOG, M, N, K, 1) (it also holds the filter
 *                re-laid as the (KH KW Cout) x C operand of that GEMM; ..._BR with log->b_r below 32).
 *   Limits: every field of the geometry below 2^24; N H W C, N Ho Wo and KH KW C below 2^31;
 *   outputs below 2^32; for VT_CONV_DATA_GRAD also N Ho Wo Cout, N H W and KH KW Cout below 2^31
 *   and KH KW below 2^16.
 */
typedef struct vt_conv2d {
    int64_t N, H, W, C;                       /* image batch, channels last */
    int64_t KH, KW;                           /* filter size */
    int64_t stride_h, stride_w, pad_h, pad_w, dil_h, dil_w;
} vt_conv2d;

#define VT_CONV_FORWARD 0
#define VT_CONV_WEIGHT_GRAD 1
#define VT_CONV_DATA_GRAD 2

int vt_conv2d_f64_round_log(int mode, const vt_conv2d *d, int64_t Cout, const double *X, const double *B,
                            const double *bias, float *C32, double *C64_debug, int variant,
                            double tau_ulp, const vt_log *log, void *ws, size_t ws_bytes, void *hip_stream);

/* The GEMM the convolution runs as: forward M = N Ho Wo, N = Cout, K = KH KW C; weight gradient
 * M = KH KW C, N = Cout, K = N Ho Wo; input gradient M = N H W, N = C, K = KH KW Cout.  Host only. */
int vt_conv2d_gemm_shape(const vt_conv2d *d, int64_t Cout, int mode, int64_t *M, int64_t *N, int64_t *K);

/*
 * The element-wise and row-wise layers of a network, fused with the trainer hook (Method: every intermediate
 * computation is rounded; Table "thresholds" lists layer norm and batch norm beside
 * convolution and linear layers).  The layer is evaluated in FP64 from its FP64 inputs and every
 * output is rounded and logged in the same pass; the FP64 output is never stored (unless asked for).
 *
 *   VT_LAYER_ADD        y = a + b                          (residual connection)
 *   VT_LAYER_RELU       y = a if a > 0, +0 otherwise (NaN stays NaN)
 *   VT_LAYER_GELU_TANH  y = a/2 (1 + tanh(sqrt(2/pi) (a + 0.044715 a^3)))
 *   VT_LAYER_GELU_ERF   y = a/2 (1 + erf(a / sqrt 2))
 *   VT_LAYER_NORM       per row: y = (a - mean) / sqrt(var + eps) * gamma + beta, biased variance;
 *                       gamma, beta per column, either may be NULL
 *   VT_LAYER_SOFTMAX    per row of z = scale * a: y = exp(z - max z) / sum exp(z - max z); with
 *                       causal_period T > 0 row r sees only columns c <= r mod T, the rest are 0
 *   VT_LAYER_BATCHNORM  training mode, per column (channel) over all rows (the N H W positions of a
 *                       channels-last activation): y = (a - mean) / sqrt(var + eps) * gamma + beta,
 *                       biased variance; VT_LAYER_BATCHNORM_RELU applies ReLU to that
 *
 *   a, b         device, rows x cols FP64, dense, 16-byte aligned
 *   y            device, rows x cols FP32, 8-byte aligned; y64_debug: optional FP64 copy of the layer
 *   variant      summation order of the row / column statistics (0 or 1), as two GPU types would differ
 *   rows * cols must be < 2^32.  ws: vt_workspace_bytes(VT_OP_LAYER_ROUND_LOG, rows, cols, 0, 1).
 */
#define VT_LAYER_ADD 0
#define VT_LAYER_RELU 1
#define VT_LAYER_GELU_TANH 2
#define VT_LAYER_GELU_ERF 3
#define VT_LAYER_NORM 4
#define VT_LAYER_SOFTMAX 5
#define VT_LAYER_BATCHNORM 6
#define VT_LAYER_BATCHNORM_RELU 7

typedef struct vt_layer {
    int32_t op;                      /* VT_LAYER_* */
    const double *a, *b;             /* b: second addend of VT_LAYER_ADD, else NULL */
    const double *gamma, *beta;      /* VT_LAYER_NORM, VT_LAYER_BATCHNORM* */
    int64_t rows, cols;
    double eps;                      /* VT_LAYER_NORM, VT_LAYER_BATCHNORM* */
    double scale;                    /* VT_LAYER_SOFTMAX */
    int64_t causal_period;           /* VT_LAYER_SOFTMAX, 0 = no mask */
} vt_layer;

int vt_layer_f64_round_log(const vt_layer *layer, float *y, double *y64_debug, int variant,
                           double tau_ulp, const vt_log *log, void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Statistics from which a per-layer threshold follows (Algorithm "threshold": the collection
 * loop over outputs y1, y2 of one layer computed on two devices; here two accumulation orders).
 *   y1, y2   device, n FP64 values each
 *   out      device, 68 x uint64:
 *            out[0]     n_flip   = #{ i : bits(rnd_32(y1[i])) != bits(rnd_32(y2[i])) }
 *            out[1]     thr_flip = 1 + max over those i of max(D(y1[i]), D(y2[i])), 0 if none:
 *                       the smallest thr that logs every observed flip, which is the value the
 *                       algorithm's binary search brackets (tau = (0.5 - (thr_flip-1) 2^-29) 2^-23)
 *            out[2]     max over i of |ord(y1[i]) - ord(y2[i])|, the distance in FP64 steps
 *            out[3+b]   histogram of that distance: b = 0 for equal, else 1 + floor(log2(distance))
 *   The call zeroes `out` itself.  Integer reductions only, so the result is order-independent.
 */
int vt_threshold_stats(const double *y1, const double *y2, uint64_t n, uint64_t *out,
                       void *hip_stream);
/* The same for rounding amount b_r (Algorithm "threshold" takes b_r as an input): rnd and D on the
 * b_r grid, thr_flip in units of 2^-29 of its spacing. */
int vt_threshold_stats_br(const double *y1, const double *y2, uint64_t n, int b_r, uint64_t *out,
                          void *hip_stream);

/*
 * Hash of the model weights at a checkpoint (Method, primitive hash_sha256(theta): a SHA-256 hash of
 * the weights in the model's precision; Algorithms "train" and "audit" append one to the Merkle
 * leaves every k steps).  The weights are hashed where they live, as the bytes in device memory.
 *
 *   chunk = 0   the SHA-256 of the whole byte string.  SHA-256 is sequential over its 64-byte blocks,
 *               so this runs on a single lane (tens of MB/s): nbytes is limited to 2^26
 *               (VT_ERR_UNSUPPORTED above); meant for small tensors and cross-checks.
 *   chunk > 0   (a multiple of 64) the same weights hashed as a tree, which is what the GPU hashes in
 *               parallel: the data is cut into chunks of `chunk` bytes (the last may be shorter),
 *               every chunk is hashed, the 32-byte digests in chunk order are the next level's data,
 *               and so on until the data fits one chunk, whose SHA-256 is the result.  Data of at
 *               most `chunk` bytes therefore gives the plain SHA-256.  Trainer and auditor must use
 *               the same chunk; it is part of what "hash" means for a run.
 *   data        device, nbytes bytes, 16-byte aligned
 *   digest      device, 32 bytes (the digest as SHA-256 prints it, first byte first), 4-byte aligned
 *   ws          at least vt_workspace_bytes(VT_OP_SHA256_TREE, 1, nbytes, chunk, 1) bytes, 256-byte aligned
 */
int vt_sha256_tree(const void *data, uint64_t nbytes, uint64_t chunk, uint8_t *digest,
                   void *ws, size_t ws_bytes, void *hip_stream);

/*
 * Root of the Merkle tree over the checkpoint hashes (Method, primitive tree(leaf_1 .. leaf_n);
 * Experimental setup: every leaf is a hash of the data and every other node a hash of its children).
 * A parent is SHA-256(left || right) over the two 32-byte children; a level's last node without a
 * sibling moves up unchanged; one leaf is its own root.
 *   leaves      device, n_leaves x 32 bytes, 4-byte aligned; n_leaves >= 1
 *   root        device, 32 bytes, 4-byte aligned
 *   ws          at least vt_workspace_bytes(VT_OP_MERKLE_ROOT, 1, n_leaves, 0, 1) bytes, 256-byte aligned
 */
int vt_merkle_root(const uint8_t *leaves, uint64_t n_leaves, uint8_t *root,
                   void *ws, size_t ws_bytes, void *hip_stream);

/* Scratch bytes needed by an operation of the given shape (0 if none). */
size_t vt_workspace_bytes(int op, int64_t M, int64_t N, int64_t K, int64_t batch);

/* ceil(tau_ulp * 2^29), or 0xFFFFFFFF if tau_ulp is not in [0, 0.5]. Host-only helper. */
uint32_t vt_thr_from_tau(double tau_ulp);

/*
 * Threshold for a layer from the statistics of its two variants (out[1] = thr_flip and out[2] =
 * max_ulp64_diff of vt_threshold_stats), in the unit of vt_thr_from_tau (tau_ulp = thr * 2^-29):
 * the smallest power of two that is at least thr_flip -- every output the two variants round
 * differently is then logged, the aim of Algorithm "threshold" -- and larger than max_ulp64_diff,
 * so that a value one party logs lies within the other party's band as well; never more than
 * VT_THR_LAYER_MAX = 2^27 (1/4 ulp, the largest threshold of Method, "Reducing storage cost"), never
 * less than 1.  Below the cap, the log written with this threshold replays without a mismatch on the
 * observed pair.  A convention of this library, not the paper's search; host arithmetic only.
 */
#define VT_THR_LAYER_MAX (1u << 27)
uint32_t vt_thr_layer_from_stats(uint64_t thr_flip, uint64_t max_ulp64_diff);

/*
 * Introspection (host only, no counterpart in the paper): the workgroup tile and the split-K
 * factor vt_gemm_f64_round_log uses for a problem of this shape and A layout: transA is
 * VT_A_ROW_MAJOR (also the forward and input-gradient views of a convolution), VT_A_TRANSPOSED (also
 * the weight gradient of a 1 x 1 convolution at every position), or VT_A_IM2COL_T (the weight
 * gradient of any other convolution).  The choice is a pure function
 * of these arguments, so a given call always accumulates in the same order.  splits > 1 (only
 * for dense outputs: ldc == N and strideC == M*N) means the K range is cut into that many
 * slices whose FP64 partial sums are added in a fixed order before the single rounding.
 */
#define VT_A_ROW_MAJOR 0
#define VT_A_TRANSPOSED 1
#define VT_A_IM2COL_T 3
int vt_gemm_plan(int transA, int64_t M, int64_t N, int64_t K, int64_t batch, int64_t ldc, int64_t strideC,
                 int *tile_m, int *tile_n, int *splits);

/*
 * Introspection (host only): when the fused path (splits = 1) launches a number of tiles a little
 * over a multiple of the 256 compute units, its last *tail_tiles tiles are each multiplied by *slices
 * workgroups (4 slices of the K range, added in slice order -- ascending for variant 0,
 * descending for variant 1 -- before the epilogue), so that the launch does not run a whole extra tile
 * time for them.  *tail_tiles = 0, *slices = 1 when it does not.  Same arguments as vt_gemm_plan; like
 * the plan, a function of the shape alone, so the accumulation order stays a function of the arguments.
 */
int vt_gemm_tail_plan(int transA, int64_t M, int64_t N, int64_t K, int64_t batch, int64_t ldc, int64_t strideC,
                      int *tail_tiles, int *slices);

/*
 * Optional instrumentation for benchmarks (no counterpart in the paper).  While two hipEvent_t
 * handles are registered, vt_gemm_f64_round_log, vt_round_log and vt_round_replay record
 * ev_begin immediately before and ev_end immediately after their MAIN kernel (the GEMM, the
 * round/decide sweep, the replay sweep) on the call's stream, so a caller can time that kernel
 * alone, without the small log-compaction kernels that follow it.  Pass NULL, NULL to clear.
 * Process-wide, not thread-safe; the events stay owned by the caller.
 */
int vt_set_kernel_events(void *ev_begin, void *ev_end);

/* Static string for a status code. */
const char *vt_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* VT_H */
