/*
 * qgbdt.h -- C ABI of the MI355X (gfx950) library for the hot path of quantized
 * GBDT training (arxiv 2207.09682): gradient quantization with stochastic
 * rounding, integer histogram construction in packed (gradient | hessian) bins,
 * sibling subtraction, best-split search, stable row partition, leaf refit and
 * the leaf-wise growth of one tree.
 *
 * Conventions
 *  - Every pointer marked "dev" is device memory owned by the caller (the Python
 *    binding hands in torch tensors); the library never frees or keeps it beyond
 *    the call's enqueued work.  Pointers marked "host" are host memory.
 *  - All work is enqueued on the context's HIP stream and is asynchronous; no
 *    entry point synchronises unless it says so.
 *  - A context belongs to the device that was current when it was created; calls on it must be
 *    made with that device current.  A context is not thread-safe: one call at a time.
 *  - Every function returns 0 (QGBDT_OK) or a negative QGBDT_E_* code;
 *    qgbdt_last_error() gives a message.  No exception crosses the boundary.
 *  - Layouts
 *      bins   uint8 (uint16 when shape.bin_bytes = 2) [n_rows][n_features], row-major,
 *             values in [0, n_bins)
 *      gh     int16 [n_rows]: quantized gradient (signed) in the high byte,
 *             quantized hessian (unsigned) in the low byte
 *      hist   int64 [n_bins][n_features] (bin-major: the order in which the kernels
 *             merge their local copies): one packed word per (bin, feature), sum of
 *             g~ in the upper 32 bits (signed), sum of h~ in the lower 32 bits
 *             (unsigned) -- the packing of Sec. 6.2 at 32|32 width
 *      rows   int32 row ids; a leaf is a contiguous slice [begin, begin+count)
 *             of an index array, ascending inside the slice
 */
#ifndef QGBDT_H
#define QGBDT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define QGBDT_API __attribute__((visibility("default")))

#define QGBDT_OK 0
#define QGBDT_E_INVALID_ARG (-1)
#define QGBDT_E_UNSUPPORTED (-2)
#define QGBDT_E_OVERFLOW_RISK (-3)
#define QGBDT_E_HIP (-4)
#define QGBDT_E_ALLOC (-5)
#define QGBDT_E_WORKSPACE (-6) /* no workspace set, the block is too small, or it lacks the section a call needs */

/* Optional sections of the workspace (qgbdt_workspace_bytes / qgbdt_set_workspace). */
#define QGBDT_WS_BIND 1u       /* feature-major copy of a bound matrix: qgbdt_bind_bins (n_rows * n_features * bin_bytes) */
#define QGBDT_WS_ROW_COPIES 2u /* three leaf-ordered copies of the bin rows: row_layout QGBDT_ROWS_ORDERED, and what
                                  QGBDT_ROWS_AUTO takes for an unbound matrix of 16..64 uint8 features (a multiple of 4);
                                  ignored for other shapes (3 * n_rows * n_features) */
#define QGBDT_WS_BOOST 4u      /* loss derivatives of qgbdt_boost_iteration* (2 * 4 bytes per row) */

#define QGBDT_ROUND_STOCHASTIC 0 /* SR of Sec. 4.2 */
#define QGBDT_ROUND_NEAREST 1    /* RN of Sec. 4.2 (half rounds up) */

/* What moves when a leaf's rows are partitioned (results are identical for all of them). */
#define QGBDT_ROWS_AUTO 0    /* ordered copies for an unbound matrix when the workspace holds them (QGBDT_WS_ROW_COPIES),
                                else row ids, with the packed gradients when the matrix is 128 MB or more */
#define QGBDT_ROWS_IDS 1     /* row ids only; histogram builds gather bin rows and packed gradients */
#define QGBDT_ROWS_IDS_GH 2  /* row ids and packed gradients; histogram builds gather the bin rows */
#define QGBDT_ROWS_ORDERED 3 /* row ids, packed gradients and bin rows: every build reads contiguous memory
                                (uint8 bins, 16..64 features that are a multiple of 4, else QGBDT_E_UNSUPPORTED;
                                needs QGBDT_WS_ROW_COPIES) */

typedef struct qgbdt_ctx qgbdt_ctx;

/* Problem shape a context is created for. */
typedef struct {
    int64_t n_rows;     /* N, 1 .. 2^31-1 */
    int32_t n_features; /* J of Algorithm 1 */
    int32_t n_bins;     /* bins per feature, 2 .. 256 (uint8 bins) or 2 .. 1024 (uint16 bins) */
    int32_t bin_bytes;  /* 1: uint8 bins; 2: uint16 bins (every `bins` argument is then uint16 [n_rows][n_features]) */
    int32_t max_leaves; /* largest num_leaves grow_tree will be asked for (at most 658: the growth
                           bookkeeping of all nodes lives in one workgroup's LDS) */
} qgbdt_shape;

/* Training parameters of one tree. */
typedef struct {
    int32_t bits_g;           /* B for gradients, 2..8 (Sec. 4.1) */
    int32_t bits_h;           /* B for hessians, 2..8; 0: the hessians are one constant and are not
                                 quantized (Sec. 4.1): every h~ is 1, delta_h is the constant */
    int32_t rounding;         /* QGBDT_ROUND_* */
    int32_t num_leaves;       /* leaf budget of leaf-wise growth */
    int32_t min_data_in_leaf; /* minimum (hessian-share estimated) rows per child */
    int32_t acc_width;        /* local accumulators: 0 auto; 16: 32-bit words (16|16 fields, or for unequal bit widths
                                 the split that takes the most rows, e.g. 13|19 for 3-bit g / 8-bit h);
                                 32: 64-bit words with 32|32 fields (Sec. 6.1, 7.4.3) */
    int32_t row_layout;       /* QGBDT_ROWS_* */
    uint64_t seed;            /* key of the counter-based RNG */
    double min_sum_hessian;   /* minimum H~ * delta_h per child */
} qgbdt_params;

/* Totals of one leaf, input of the split search. */
typedef struct {
    int64_t n_rows;
    int64_t sum_g; /* G~_s */
    int64_t sum_h; /* H~_s */
} qgbdt_leafstat;

/* Best split of one leaf; feature = -1 (gain 0) when no candidate is valid. */
typedef struct {
    double gain; /* eq. (gain) of Sec. 4.1, fp64 */
    int32_t feature;
    int32_t bin; /* rows with bin <= this go left */
    int64_t left_g, left_h, right_g, right_h;
    int64_t left_count; /* hessian-share estimate, rounded half up */
} qgbdt_split;

/* Output of grow_tree: device arrays, all caller-allocated.
 * split_* are in split order (entry k is the k-th split), leaf_* by leaf id. */
typedef struct {
    int32_t* n_leaves;        /* dev[1] */
    int32_t* split_leaf;      /* dev[max_leaves-1] id of the leaf that was split */
    int32_t* split_feature;   /* dev[max_leaves-1] */
    int32_t* split_bin;       /* dev[max_leaves-1] */
    double* split_gain;       /* dev[max_leaves-1] */
    int64_t* split_stats;     /* dev[(max_leaves-1)*4] left_g, left_h, right_g, right_h */
    int64_t* split_n_left;    /* dev[max_leaves-1] true number of rows sent left */
    int64_t* leaf_begin;      /* dev[max_leaves] slice of row_idx_out */
    int64_t* leaf_count;      /* dev[max_leaves] */
    int64_t* leaf_sum_g;      /* dev[max_leaves] G~ of the leaf */
    int64_t* leaf_sum_h;      /* dev[max_leaves] H~ of the leaf */
    double* leaf_value;       /* dev[max_leaves] refit with FP gradients, eq. (leaf) */
    double* leaf_value_quant; /* dev[max_leaves] -G~ delta_g / (H~ delta_h), Sec. 4.2 */
    float* delta;             /* dev[2] delta_g, delta_h */
    int64_t* hist_units;      /* dev[1] sum over histogram builds of rows*features accumulated */
} qgbdt_tree;

/* ---- lifecycle ---------------------------------------------------------- */

/* Device memory: the caller owns all of it.  The library allocates no device memory anywhere; it owns only the
 * host-side context (and a few bytes of pinned host memory for the status word grow_tree reads back).
 *
 * qgbdt_workspace_bytes: bytes of device workspace a context of `shape` needs (host out), from the shape alone:
 * three row-index buffers and three lists of packed gradients that follow them, the quantized gradients, a pool of
 * 3 * max_leaves + 1 histograms, the slots of the histogram kernels' row groups, partition flags and small
 * descriptors, plus the optional sections named by `flags` (QGBDT_WS_*).
 *
 * qgbdt_create: a context for `shape` on the current device; `stream` is a hipStream_t (NULL = default stream).
 * Allocates no device memory; tells the runtime once which kernels need more than the default dynamic LDS.
 *
 * qgbdt_set_workspace: hands the context a block `dev` (device memory, 256-byte aligned, at least
 * qgbdt_workspace_bytes(shape, flags) bytes; QGBDT_E_WORKSPACE if smaller) that it carves all its buffers from.
 * The block stays the caller's: it must live until the context is destroyed or given another block, and nothing
 * else may write it meanwhile.  Synchronises the stream (earlier work may use the previous block), then enqueues
 * a few bytes of initialisation.  A bound matrix is forgotten.  dev = NULL detaches the block.  Every step
 * returns QGBDT_E_WORKSPACE while no block is set, or when it needs an optional section the block was set without. */
QGBDT_API int qgbdt_workspace_bytes(const qgbdt_shape* shape, uint32_t flags, size_t* bytes);
QGBDT_API int qgbdt_create(qgbdt_ctx** out, const qgbdt_shape* shape, void* stream);
QGBDT_API int qgbdt_set_workspace(qgbdt_ctx* ctx, void* dev, size_t bytes, uint32_t flags);
/* Frees the context (never the workspace).  Synchronises the stream first. */
QGBDT_API int qgbdt_destroy(qgbdt_ctx* ctx);
/* Changes the stream later calls enqueue on. */
QGBDT_API int qgbdt_set_stream(qgbdt_ctx* ctx, void* stream);
/* Message of the last error on this context (or of a failed create / workspace_bytes when ctx is NULL). */
QGBDT_API const char* qgbdt_last_error(const qgbdt_ctx* ctx);

/* Optional.  Declares that `bins` (dev) is the matrix of the grow_tree / boost_iteration calls that follow,
 * as it is for all trees of a boosting run, and makes a feature-major copy of it on the stream
 * (in the QGBDT_WS_BIND section of the workspace; QGBDT_E_WORKSPACE without it).  The counting pass of
 * the row partition then reads the split feature's column -- the ascending row ids of a node fall into
 * few memory sectors -- instead of one sector of the row-major matrix per row, and narrow matrices, whose
 * rows are otherwise moved into leaf order level by level, are left in place.  The call also samples the
 * columns for each feature's most frequent bin; when most features have a bin that holds most of their rows,
 * the wide-row histogram kernels leave that bin out and the entry is rebuilt from the totals.  Results do not
 * change.
 * Call again after the matrix' contents change; a grow_tree call with another pointer simply does not
 * use the copy; bins = NULL forgets the matrix. */
QGBDT_API int qgbdt_bind_bins(qgbdt_ctx* ctx, const void* bins);

/* ---- steps of the path ---------------------------------------------------- */

/* Sec. 4.1 (interval lengths, eq. (scale)) and Sec. 4.2 (SR / RN).
 * delta_g = max|g| / (2^(bits_g-1)-1), delta_h = max h / (2^bits_h-2) over all n rows,
 * then g~ = Round(g/delta_g) in [-(2^(bits_g-1)-1), ..], h~ = Round(h/delta_h) in
 * [0, 2^bits_h-2], fp32 arithmetic.  Stochastic rounding draws its uniform numbers
 * from Philox-4x32-10 keyed by `seed` with counter (row, iteration): output word 0
 * rounds g, word 1 rounds h, top 24 bits each.  g, h: dev float[n]; gh_out: dev
 * int16[n]; delta_out: dev float[2].  n <= shape.n_rows.  bits_h = 0 (constant hessians,
 * the caller's precondition): h~ = 1 for every row and delta_h = max h. */
QGBDT_API int qgbdt_quantize_gradients(qgbdt_ctx* ctx, const float* g, const float* h, int64_t n,
                             int32_t bits_g, int32_t bits_h, uint64_t seed, uint32_t iteration,
                             int32_t rounding, int16_t* gh_out, float* delta_out);

/* Algorithm 1 with quantized gradients (Sec. 4.1), accumulated in workgroup-local
 * packed low-width bins and merged into the total histogram (Sec. 6.1, 6.2).
 * Rows are row_idx[begin .. begin+count) (dev int32) or, when row_idx is NULL,
 * begin .. begin+count.  bits_g/bits_h bound |g~|, h~ and set how many rows a local
 * 32-bit accumulator word may take before it is merged (Sec. 7.4.3); acc_width 0 picks the
 * width, 16 (32-bit words) / 32 (64-bit words) force it.  hist_out: dev int64[n_bins][n_features], overwritten.
 * QGBDT_E_OVERFLOW_RISK if count rows could overflow a 32-bit field. */
QGBDT_API int qgbdt_build_histograms(qgbdt_ctx* ctx, const void* bins, const int16_t* gh,
                           const int32_t* row_idx, int64_t begin, int64_t count, int32_t bits_g,
                           int32_t bits_h, int32_t acc_width, int64_t* hist_out);

/* sibling = parent - child, bin by bin on the packed words (exact: a child's sums
 * never exceed its parent's).  All dev int64[n_bins][n_features]; sibling_out may
 * alias parent. */
QGBDT_API int qgbdt_subtract_histograms(qgbdt_ctx* ctx, const int64_t* parent, const int64_t* child,
                              int64_t* sibling_out);

/* Best split of each of n_hists leaves: thresholds of every feature enumerated
 * (Sec. 3), integer prefix sums, fp64 gain of eq. (gain) (Sec. 4.1).  A candidate
 * needs H~ > 0 on both sides, both estimated row counts >= min_data_in_leaf and both
 * H~ delta_h >= min_sum_hessian; the strictly largest gain > 0 wins, ties go to the
 * lowest feature, then the lowest bin.  hist: dev int64[n_hists][nb][F]; stats: dev
 * [n_hists]; delta: dev float[2]; out: dev [n_hists]. */
QGBDT_API int qgbdt_find_best_splits(qgbdt_ctx* ctx, const int64_t* hist, int32_t n_hists,
                           const qgbdt_leafstat* stats, const float* delta,
                           int32_t min_data_in_leaf, double min_sum_hessian, qgbdt_split* out);

/* The same search for callers that cannot allocate or be handed a workspace: code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation.  Works on a context with no workspace set and calls no
 * allocating routine.  Its scratch (one item per histogram, one candidate per (histogram, feature)) lives in a
 * fixed array of 4 MiB inside the library, of which every GPU the library runs on holds its own copy until the
 * process ends: n_hists * (48 + 24 * n_features) + 512 bytes must fit (about 5,800 histograms of 28 features, 87 of
 * 2000), else QGBDT_E_INVALID_ARG.  All calls on one GPU share that array and nothing in it needs clearing between
 * calls (every entry a call reads it has written before); calls that overlap on one GPU -- two streams, two
 * contexts, two threads -- race on it.  Arguments and results as qgbdt_find_best_splits. */
QGBDT_API int qgbdt_find_best_splits_static(qgbdt_ctx* ctx, const int64_t* hist, int32_t n_hists,
                                  const qgbdt_leafstat* stats, const float* delta,
                                  int32_t min_data_in_leaf, double min_sum_hessian, qgbdt_split* out);

/* Stable partition of the slice row_idx[begin..begin+count) (the set I_s of
 * Algorithm 1): rows with bins[row][feature] <= bin first, both sides keeping their
 * order.  row_idx: dev int32, reordered in place; n_left_out: dev int64[1]. */
QGBDT_API int qgbdt_partition_rows(qgbdt_ctx* ctx, const void* bins, int32_t* row_idx, int64_t begin,
                         int64_t count, int32_t feature, int32_t bin, int64_t* n_left_out);

/* Leaf values from the original FP gradients (eq. (leaf) of Sec. 3, refit of
 * Sec. 4.2): value[l] = -sum g / sum h over row_idx[leaf_begin[l] .. +leaf_count[l]),
 * fp64 sums; 0 when sum h <= 0.  leaf_begin, leaf_count: dev int64[n_leaves];
 * value_out: dev double[n_leaves]. */
QGBDT_API int qgbdt_refit_leaves(qgbdt_ctx* ctx, const float* g, const float* h, const int32_t* row_idx,
                       const int64_t* leaf_begin, const int64_t* leaf_count, int32_t n_leaves,
                       double* value_out);

/* One tree, leaf-wise (Sec. 3, Sec. 7): quantize (g,h), build the root histogram,
 * then repeatedly split the open leaf with the largest gain (ties: lowest id); the
 * left child keeps the parent's id, the right child takes the next id; the child
 * with fewer rows (tie: left) is built from its rows, its sibling by subtraction;
 * stops at num_leaves or when no gain > 0 is left; leaf values are refit at the end.
 * The result is that of this sequential procedure; the work is done in rounds that
 * expand several leaves at once (the one the procedure needs next plus leaves it is
 * likely to need), and the order of the splits is replayed on the device.  The host
 * waits on the stream once per batch of rounds to read a 'finished' flag (normally
 * once per tree) and, when n_rows exceeds what a 32-bit field surely holds, once
 * more after quantization to check the quantized totals (QGBDT_E_OVERFLOW_RISK).
 * bins: dev; g, h: dev float[n_rows]; row_idx_out: dev int32[n_rows], leaf-ordered
 * rows (ascending inside each leaf). */
QGBDT_API int qgbdt_grow_tree(qgbdt_ctx* ctx, const void* bins, const float* g, const float* h,
                    const qgbdt_params* params, uint32_t iteration, const qgbdt_tree* tree_out,
                    int32_t* row_idx_out);

/* ---- around the tree: one boosting iteration on the device ------------------ */

/* g_i, h_i = first and second derivative of the loss w.r.t. the current prediction (Sec. 3)
 * for the binary cross-entropy loss: p = 1/(1+exp(-score)), g = p - label, h = p (1 - p),
 * evaluated in fp64 and rounded once to fp32.  All dev float[n]; n <= shape.n_rows. */
QGBDT_API int qgbdt_logistic_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n,
                             float* g_out, float* h_out);

/* The same for the pairwise ranking loss with NDCG weights (lambdarank, the objective of the
 * paper's ranking experiments, Sec. 7).  Rows form consecutive queries of group_size rows (the
 * last may be shorter); relevance holds integer grades.  Inside a query documents are ranked by
 * score, descending, ties by position; gain = 2^rel - 1, discount = 1/log2(rank+2), maxDCG the
 * DCG of the gains in descending order.  Every pair (a, b) with rel_a > rel_b contributes
 * rho = 1/(1+exp(s_a-s_b)), w = |gain_a-gain_b| |disc_a-disc_b| / maxDCG:  g_a -= rho w,
 * g_b += rho w, h_a and h_b += rho (1-rho) w.  fp64, rounded once to fp32.  1 <= group_size <= 1024. */
QGBDT_API int qgbdt_lambdarank_gradients(qgbdt_ctx* ctx, const float* score, const float* relevance, int64_t n,
                               int32_t group_size, float* g_out, float* h_out);

/* Prediction update with a tree (Sec. 3; the learning rate scales the leaf values):
 * score[row] += (float)(learning_rate * leaf_value[l]) for the rows of every leaf l, one fp32
 * addition per row.  Leaves are slices of the leaf-ordered row list as grow_tree returns
 * them.  score: dev float[n_rows], updated in place; leaf_begin, leaf_count: dev int64
 * [n_leaves]; leaf_value: dev double[n_leaves]. */
QGBDT_API int qgbdt_update_scores(qgbdt_ctx* ctx, float* score, const int32_t* row_idx, const int64_t* leaf_begin,
                        const int64_t* leaf_count, const double* leaf_value, int32_t n_leaves,
                        double learning_rate);

/* One boosting iteration for the binary cross-entropy loss without any host arithmetic:
 * loss derivatives of `score`, one tree (qgbdt_grow_tree with these derivatives), score
 * update with learning_rate times the refit leaf values.  label: dev float[n_rows] (0 / 1);
 * score: dev float[n_rows], updated in place; the rest as in qgbdt_grow_tree.  The derivatives
 * live in the QGBDT_WS_BOOST section of the workspace (QGBDT_E_WORKSPACE without it). */
QGBDT_API int qgbdt_boost_iteration(qgbdt_ctx* ctx, const void* bins, const float* label, float* score,
                          const qgbdt_params* params, uint32_t iteration, double learning_rate,
                          const qgbdt_tree* tree_out, int32_t* row_idx_out);

/* One boosting iteration for the lambdarank loss (qgbdt_lambdarank_gradients, then as above). */
QGBDT_API int qgbdt_boost_iteration_lambdarank(qgbdt_ctx* ctx, const void* bins, const float* relevance,
                                     int32_t group_size, float* score, const qgbdt_params* params,
                                     uint32_t iteration, double learning_rate, const qgbdt_tree* tree_out,
                                     int32_t* row_idx_out);

/* ---- measurement ---------------------------------------------------------- */

/* When on, every histogram-kernel launch is bracketed by HIP events on the
 * context's stream. */
QGBDT_API int qgbdt_set_profiling(qgbdt_ctx* ctx, int32_t on);
/* Synchronises the stream, returns the summed histogram-kernel time (ms), the
 * number of launches and their summed algorithmic bytes since the last call, and
 * resets the counters (host out pointers). */
QGBDT_API int qgbdt_read_profile(qgbdt_ctx* ctx, double* hist_ms, int64_t* hist_launches,
                       double* hist_bytes);

/* Of the launches timed since the last qgbdt_read_profile: the summed time (ms) and the number of those that
 * were a tree's root build inside qgbdt_grow_tree (all rows, contiguous; its algorithmic bytes are
 * n_rows * (n_features * bin_bytes + 2) + n_features * n_bins * 8 per launch).  Synchronises the stream; resets
 * nothing, so call it before qgbdt_read_profile.  Host out pointers. */
QGBDT_API int qgbdt_read_profile_roots(qgbdt_ctx* ctx, double* root_ms, int64_t* root_launches);

/* The launch plan the histogram kernels would be given for a shape (host-only: no context, no GPU call), for
 * callers and tests that check the plan against its invariants.  rows / n_builds: the rows a launch serves and
 * the number of builds they belong to (1 with rows > 0: a stand-alone build of that many contiguous rows of a
 * 16-byte aligned matrix).  out (host int64 [25]): features per tile, tile pitch in LDS words, dwords per tile row, rows per wavefront step, feature tiles,
 * threads per workgroup, bytes of local bins, rows per chunk (width rule of Sec. 7.4.3), row groups of one build,
 * row-group lanes of a launch, least rows per group, word width of the local bins (16: 32-bit words, 32: 64-bit),
 * bits of the hessian field of a 32-bit word, lanes / rows per step of the byte-stream kernel (0: not used), most
 * work items of a launch, bytes of a row group's slot, most rows of a one-chunk group, padded pitch flag, bytes per
 * lane of the wide-row kernels (0: not used), unaligned-row flag, element-wise flag, rows per row group for
 * (rows, n_builds), bytes of the workspace section that holds the slots, two-level flag (32-bit working words folded
 * into 64-bit words in LDS after every chunk: the slots then hold 64-bit words). */
QGBDT_API int qgbdt_describe_hist_plan(const qgbdt_shape* shape, int32_t bits_g, int32_t bits_h, int32_t acc_width,
                             int32_t skewed, int64_t rows, int32_t n_builds, int64_t* out, int32_t n_out);

/* Figures of the last grow_tree call on this context (host out int32[4]): rounds of
 * batched expansion, nodes expanded (committed splits plus speculative ones), committed
 * splits, nodes created.  For callers that time or tune; no paper quantity. */
QGBDT_API int qgbdt_tree_stats(const qgbdt_ctx* ctx, int32_t* out4);

/* Streaming-read rate of this device as a plain kernel reaches it: `buf` (dev, 16-byte aligned, `bytes` a
 * multiple of 16, at least 16) is read `reps` times with 16-byte loads by one grid-stride kernel per repetition,
 * timed with HIP events on the context's stream after one untimed repetition -- for every combination of 4, 8 or
 * 16 loads in flight per thread, 4 to 32 workgroups of 256 threads per compute unit, and plain or non-temporal
 * loads; the best rate is returned.  gbps_out (host) = bytes * reps / time in GB/s; variant_out (host int32[3],
 * may be NULL) = loads in flight, workgroups and 1 for non-temporal loads of the best run.  Synchronous.  The
 * measured ceiling that the histogram kernels' rates are set against beside the published peak; no paper
 * quantity. */
QGBDT_API int qgbdt_measure_stream_read(qgbdt_ctx* ctx, const void* buf, int64_t bytes, int32_t reps, double* gbps_out,
                              int32_t* variant_out);

#ifdef __cplusplus
}
#endif
#endif /* QGBDT_H */
