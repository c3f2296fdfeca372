// vt_kernels.h -- host-callable launchers of the gfx950 kernels (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace vt {

// A "segment" is 64 consecutive 64-bit words of a decision bit-plane (4096 outputs); one
// wavefront owns one segment in the plane-producing and plane-compacting kernels.
constexpr uint32_t kSegWords = 64;
constexpr uint32_t kSegElems = 64 * kSegWords;

// Decision bit-planes and per-segment bookkeeping inside the caller's workspace.
struct Planes {
    uint64_t *logged;    // [segs * 64] bit = 1: output is logged
    uint64_t *dir;       // [segs * 64] bit = 1: rounded toward +inf
    uint32_t *seg_cnt;   // [segs] logged outputs per segment
    uint32_t *seg_off;   // [segs] exclusive prefix of seg_cnt
    uint64_t words;      // words in use (rows * words_per_row)
    uint32_t segs;       // ceil(words / 64)
    // bit -> linear index mapping: word w covers row w / wpr, columns 64 * (w % wpr) ...
    uint32_t wpr;        // words per row
    uint32_t ncols;      // row length N (linear index = row * N + col)
};

size_t planes_bytes(uint64_t rows, uint64_t ncols);
Planes planes_carve(void *ws, uint64_t rows, uint64_t ncols);

struct LogOut {
    uint32_t *idx;
    uint32_t *dir;
    uint64_t cap;
    uint64_t *count;
};

// round + decide on a flat array: y, both bit-planes and seg_cnt (standalone trainer hook)
// (k = 32 - b_r low mantissa bits of every FP32 result are zero; 0 is plain FP32, see vt_device.h)
hipError_t launch_round_planes(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, const Planes &pl,
                               hipStream_t s);
// seg_cnt from an already written `logged` plane (GEMM epilogue output)
hipError_t launch_seg_count(const Planes &pl, hipStream_t s);
// seg_off = exclusive scan(seg_cnt); *count = total; clears the dir words compaction will OR into
hipError_t launch_seg_scan(const Planes &pl, const LogOut &log, hipStream_t s);
// ordered stream compaction: planes -> ascending idx[] + packed direction bits
hipError_t launch_compact(const Planes &pl, const LogOut &log, hipStream_t s);

// The three kernels above as one launch (a scanner workgroup hands the tiles their offsets).  Needs zeroed
// beforehand, by the kernel that wrote the planes: the scratch that compact_onepass_scratch names (inside
// the planes' bookkeeping arrays) and the first ceil(min(cap, outputs) / 32) direction words of the log.
void compact_onepass_scratch(const Planes &pl, uint32_t **zero, uint32_t *zero_words);
hipError_t launch_compact_onepass(const Planes &pl, const LogOut &log, hipStream_t s);

// single-pass standalone trainer hook (chained scan); needs x 16-byte and y 8-byte aligned
size_t onepass_bytes(uint64_t n);
bool onepass_usable(const double *x, const float *y);
hipError_t launch_round_log_onepass(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s);

// threshold 0 (nothing is logged): y = rnd(x), *count = 0, as one plain stream; same alignment as the single-pass kernel
hipError_t launch_round_only(const double *x, uint64_t n, uint32_t k, float *y, uint64_t *count, hipStream_t s);

hipError_t launch_replay(const double *x, uint64_t n, const uint32_t *idx, const uint32_t *dir,
                         uint64_t count, uint32_t k, float *y, hipStream_t s);

// the paper's packed ternary log (five entries per byte): trainer, auditor, and from bit-planes
size_t dense_count_bytes();   // scratch for the logged-output count of the call below
hipError_t launch_round_log_dense(const double *x, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s);
hipError_t launch_replay_dense(const double *x, uint64_t n, const uint8_t *tlog, uint32_t k, float *y, hipStream_t s);
hipError_t launch_planes_to_dense(const Planes &pl, uint64_t rows, uint8_t *tlog, uint64_t *count, hipStream_t s);

// ---- element-wise and row-wise layers fused with the trainer hook -----------------------------
// Layer selectors (the public VT_LAYER_* values).
enum { kLayerAdd = 0, kLayerRelu = 1, kLayerGeluTanh = 2, kLayerGeluErf = 3, kLayerNorm = 4, kLayerSoftmax = 5,
       kLayerBatchNorm = 6, kLayerBatchNormRelu = 7 };

struct LayerArgs {
    int op;
    const double *a, *b;          // inputs (b: second addend of the residual add)
    const double *gamma, *beta;   // layer norm: per-column scale and shift, either may be null
    const double *stat;           // per row: (mean, 1/std) for layer norm, (max, 1/sum) for softmax;
                                  // per column: (mean, 1/std) for batch norm
    double *y64;                  // optional FP64 copy of the layer's output
    uint32_t cols;
    double inv_cols;              // 1 / cols (index split by reciprocal multiply + correction)
    double scale;                 // softmax: logits are scale * a
    uint32_t period;              // softmax: causal mask period, 0 = none
    double inv_period;
    double eps;                   // layer norm, batch norm
    int variant;                  // summation order of the statistics
};

size_t layer_stat_bytes(uint64_t rows, uint64_t cols);
// per-row statistics of layer norm / softmax, per-column statistics of batch norm into g.stat
// (no-op for the element-wise layers; batch norm also uses the scratch that follows g.stat);
// g.variant selects the summation order
hipError_t launch_layer_stats(const LayerArgs &g, uint64_t rows, hipStream_t s);
// Layer norm and softmax a row at a time in registers (vt_round_rowwise.hip): one read of the input,
// softmax with one exponential per value.  Rows of 64 to 1024 columns (a row of 2048 in registers
// measured slower than the two passes: 1.34 against 1.09 ms for layer norm over 2^28 values); other
// row lengths take the statistics kernel and the element-wise pass.  Same bits either way.
constexpr uint32_t kRowwiseMinCols = 64, kRowwiseMaxCols = 1024;
bool rowwise_usable(int op, uint64_t cols);
size_t rowwise_bytes(uint64_t rows);      // scratch of launch_rowwise_onepass
hipError_t launch_rowwise_dense(const LayerArgs &g, uint64_t rows, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                uint64_t *n_logged, uint64_t *slots, hipStream_t s);
hipError_t launch_rowwise_onepass(const LayerArgs &g, uint64_t rows, uint32_t thr, uint32_t k, float *y, void *ws,
                                  const LogOut &log, hipStream_t s);
// shared by the kernels that write the packed log: clear the spread counters (or *n_logged when
// slots is null and n_logged is not) before the pass, fold them into *n_logged after it
hipError_t launch_count_begin(uint64_t *slots, uint64_t *n_logged, hipStream_t s);
hipError_t launch_count_end(const uint64_t *slots, uint64_t *n_logged, hipStream_t s);
// shared by the single-pass index-list kernels: status words, error words, direction words, count
hipError_t launch_onepass_init(uint64_t *st, uint32_t tiles, uint32_t *err, const LogOut &log, uint64_t n, hipStream_t s);
hipError_t launch_layer_log_onepass(const LayerArgs &g, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s);
hipError_t launch_layer_log_dense(const LayerArgs &g, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s);

// SHA-256 of a byte string as a tree of chunks (chunk 0: the plain, sequential hash) and the
// Merkle root over 32-byte leaves; digests are 32 bytes in device memory, 4-byte aligned
size_t sha256_tree_bytes(uint64_t nbytes, uint64_t chunk);
hipError_t launch_sha256_tree(const uint8_t *data, uint64_t nbytes, uint64_t chunk, uint32_t *digest, void *ws,
                              hipStream_t s);
size_t merkle_root_bytes(uint64_t n_leaves);
hipError_t launch_merkle_root(const uint32_t *leaves, uint64_t n_leaves, uint32_t *root, void *ws, hipStream_t s);

// the trainer hook over the result of a split-K GEMM, summed from its slabs on the fly (slab even,
// y 8-byte aligned, y64 null or 16-byte aligned); same outputs as the two calls above on the sum
struct SplitKArgs {
    const double *partial; uint64_t slab; int splits, variant; double alpha; const double *bias; uint32_t ncols;
    double *y64;
};
hipError_t launch_splitk_log_onepass(const SplitKArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                     const LogOut &log, hipStream_t s);
hipError_t launch_splitk_log_dense(const SplitKArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                   uint64_t *n_logged, uint64_t *slots, hipStream_t s);

// the trainer hook over an input gradient computed phase by phase (see PhaseSource in vt_source.h;
// C even, slabs 16-byte aligned, y 8-byte aligned, y64 null or 16-byte aligned)
struct PhaseArgs {
    const double *P;
    uint32_t H, W, C, ph, pw, sh, sw;       // sh, sw: 1 or 2
    uint32_t q0h[2], Ha[2], q0w[2], Wb[2], off[4], has;
    double *y64;
};
hipError_t launch_phase_log_onepass(const PhaseArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, void *ws,
                                    const LogOut &log, hipStream_t s);
hipError_t launch_phase_log_dense(const PhaseArgs &a, uint64_t n, uint32_t thr, uint32_t k, float *y, uint8_t *tlog,
                                  uint64_t *n_logged, uint64_t *slots, hipStream_t s);

hipError_t launch_stats(const double *y1, const double *y2, uint64_t n, uint32_t k, uint64_t *out, hipStream_t s);

// Geometry of a channels-last convolution whose image the GEMM kernel reads through an implicit
// im2col view (all sizes already validated by the caller).
struct ConvDesc {
    int64_t N, H, W, C, KH, KW, stride_h, stride_w, pad_h, pad_w, dil_h, dil_w, Ho, Wo;
};

struct GemmArgs {
    const ConvDesc *conv = nullptr;   // non-null: A is an image X[N][H][W][C]; M, K describe its im2col matrix
    bool conv_wgrad = false;          // the matrix is used transposed (taps x rows): weight gradient
    int64_t conv_dgrad_cout = 0;      // > 0: A is the output gradient dY[N][Ho][Wo][Cout] read through the
                                      // input-gradient view (rows = input positions, K = KH KW Cout)
    int transA, transB;
    int64_t M, N, K;
    double alpha;
    const double *A; int64_t lda, strideA;
    const double *B; int64_t ldb, strideB;
    const double *bias;
    int64_t batch;
    int64_t batch_inner = 0;          // > 0: matrix b = (group b / batch_inner, member b % batch_inner); groups are
    int64_t strideA2 = 0, strideB2 = 0;   // strideA2 / strideB2 apart, members strideA / strideB
    float *C32; int64_t ldc, strideC;
    double *C64;          // optional dense FP64 copy (pitch N)
    int variant;
    uint32_t thr;
    bool raw = false;     // leave alpha, bias and the rounding to a later pass even without split-K
    // two arrays of 32-bit words the kernel clears on its way (what the log compaction that follows needs zeroed)
    uint32_t *zero_a = nullptr, *zero_b = nullptr;
    uint32_t zero_a_words = 0, zero_b_words = 0;
    // scratch for the slices of tail tiles (tiles % 256 x 4 slices x tile area, in doubles; 256-byte aligned), or
    // null: lets the launcher share the last few tiles of a launch whose tile count is a little over a multiple
    // of the compute units among several workgroups (gemm_tail_cut)
    double *tail_ws = nullptr;
};
bool gemm_tail_cut(int shape, uint64_t tiles, int64_t nkt);   // the last tiles % 256 tiles are cut into four slices of K
// Tile shape (index into the kernel's shape table) and split-K factor chosen for a problem.
struct GemmPlan {
    int shape;          // 0: 128x128, 1: 64x64
    int splits;         // 1 = fused epilogue; > 1 = slabs + fixed-order reduction + round/log pass
    int kt_per_split;   // k steps of 16 per slice
};
// a_layout: how the A operand reaches the kernel (the public VT_A_* values)
enum { kALayoutRowMajor = 0, kALayoutTransposed = 1, kALayoutIm2colT = 3 };
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t K, int64_t batch, bool allow_split, int a_layout);
size_t gemm_split_bytes(int64_t M, int64_t N, int64_t batch, int splits);
// splits == 1 and not g.raw: C32 / C64 / planes written by the epilogue.  Otherwise `partial`
// receives the slabs, `reduced` (and g.C64 if set) the FP64 result alpha * sum + bias; nothing
// else is written.  With `reduced` null only the slabs are written (the caller sums them where it
// consumes them).
hipError_t launch_gemm_round_planes(const GemmArgs &g, const GemmPlan &plan, const Planes &pl, double *partial,
                                    double *reduced, hipStream_t s);
// up to four problems (raw accumulators to partial[i]; no split-K, no planes) of tile shape `shape` in one launch
hipError_t launch_gemm_group(const GemmArgs *g, double *const *partial, int count, int shape, hipStream_t s);
// Filter Wt[KH][KW][C][Cout] -> Wp[filter position][Cout][C]: the B operand (K x C, row-major) of the
// input-gradient GEMM.  A copy, so exact.
// Only the filter positions (kh0 + sth i, kw0 + stw j), i < nkh, j < nkw, are taken (a stride phase's
// sub-filter); the whole filter is (0, 1, KH, 0, 1, KW).
hipError_t launch_dgrad_weights(const double *Wt, int64_t KW, int64_t C, int64_t Cout, int64_t kh0, int64_t sth, int64_t nkh,
                                int64_t kw0, int64_t stw, int64_t nkw, double *Wp, hipStream_t s);

}  // namespace vt
