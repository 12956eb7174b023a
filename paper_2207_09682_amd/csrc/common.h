// Internal declarations shared by the HIP translation units of libqgbdt.
// Nothing here is part of the public boundary (see include/qgbdt.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/qgbdt.h"

namespace qgbdt {

// ---- device-side bookkeeping of one tree -----------------------------------

// A node of the tree being grown.  Nodes are created in pairs when their parent is
// expanded (partitioned, histograms built, best split searched); a node becomes an
// open leaf when its parent's split is committed in best-first order.
struct Node {
    int64_t begin, count;  // slice of the index buffer `buf`
    int64_t sum_g, sum_h;  // quantized totals
    int64_t n_left;        // rows sent left by this node's split (valid once expanded)
    int32_t buf;           // which of the two index buffers holds the slice
    int32_t slot;          // histogram slot in the pool
    int32_t state;         // 0 waiting for its parent's commit, 1 open leaf, 2 internal (split committed)
    int32_t expanded;      // children exist (their rows, histograms and best splits are known)
    int32_t child;         // left child id (right = child + 1), -1 if none
    int32_t leaf_id;       // valid once the node is an open leaf
    qgbdt_split best;      // best split of this node (feature < 0: none)
};

// State of the growth of one tree.
struct StepState {
    int32_t done;        // 1: tree finished, later kernels return at once
    int32_t n_nodes, n_leaves, n_commits, n_expanded, n_slots;
    int32_t n_batch;     // nodes expanded in the current round
    int32_t rounds;
    int32_t n_part_items;  // row segments of the current round's partitions
    int32_t n_scan_items;  // histograms to scan in the current round
    int32_t n_sorted;      // nodes in the kept gain order (see tree_plan_kernel)
    int32_t pad[1];
    int64_t hist_units;    // rows*features of the histogram builds the sequential algorithm performs
    int64_t prof_rows_contig, prof_rows_idx;  // rows seen by histogram launches
    int64_t prof_launches;                    // histogram launches that had rows
    int64_t prof_builds;                      // histogram builds served by those launches
};

// One node expanded in the current round.
struct BatchEntry {
    int32_t node;
    int32_t seg_start;  // first partition segment of this node
    int32_t n_seg;
    int32_t new_slot;   // histogram slot of the child that is built from its rows
};

// Candidate of one (leaf, feature) pair produced by the scan kernel.
struct FeatCand {
    double gain;
    int64_t left;  // packed prefix word (G_L | H_L)
    int32_t bin;   // -1: no valid candidate
    int32_t pad;
};

// One histogram build: a row slice accumulated into one slot, cut into `groups` row groups
// that are the work items [item_start, item_start + groups) of the launch.
struct HistEntry {
    int64_t begin, count;
    int32_t buf;   // index buffer (gathered builds)
    int32_t slot;  // histogram slot relative to the base pointer
    int32_t item_start;
    int32_t groups;
};

// Work descriptor of one stand-alone row partition.
struct PartWork {
    int64_t begin, count;
    int32_t feature, bin;
    int32_t src_buf;    // which index buffer holds the slice; the result goes to the other one
    int32_t zero_slot;  // unused by the stand-alone call
};

struct HistPlan {
    int32_t ft;          // features per workgroup tile (a multiple of 4 unless the tile is the whole row)
    int32_t ftp;         // padded tile width in LDS words
    int32_t dpr;         // dwords per row per tile = ceil(ft/4)
    int32_t rows_per_it; // rows one wavefront covers per iteration
    int32_t n_tiles;     // feature tiles
    int32_t threads;     // workgroup size
    int32_t lds_bytes;
    int32_t chunk_rows;  // rows accumulated between two merges of the local bins
    int32_t max_groups;  // row groups of one build: all its workgroups are resident at once
    int32_t max_lanes;   // workgroups along the row axis of a launch with many builds (a multiple of 8)
    int32_t min_rows_per_group;
    int32_t acc_width;   // 16: packed 32-bit words in LDS (g~ sums above hshift, h~ sums below), 32: packed 32|32 words
    int32_t hshift;      // bits of the hessian field of a 32-bit local word: 16, or the split that takes more rows
    int32_t flat_lanes;  // > 0: contiguous slices may use the flat 16-byte-load kernel with this many lanes
    int32_t flat_rows;   // rows per wavefront iteration of that kernel
    int32_t flat_unroll;
    int32_t max_items;    // most work items (row groups) of one launch = slots of the partial-histogram buffer
    int32_t slot_bytes;   // bytes of one (item, tile) slot: the tile's local bins, padded to 16 bytes
    int32_t single_rows;  // a group of at most this many rows is accumulated in one chunk by every kernel variant
    int32_t pad16;        // local bins keep 4 unused words after every 16 features (wide rows, 16-byte loads)
    int32_t wide_v;       // > 0: wide rows are read in pieces of this many bytes per lane (8 or 16)
    int32_t ragged;       // feature count not a multiple of 4: unaligned dword loads, last dword of a tile row partial
    int32_t bytewise;     // no dword kernel applies (rows or a tile narrower than 4 bytes): one byte load per bin
    int32_t two_level;    // byte-stream kernel with 32-bit working words folded into 64-bit words in LDS after every chunk
                          // (one large contiguous build: few, long row groups; slots hold the 64-bit words)
};

// Rows per row group when `total` rows of `n_entries` builds are shared out: about max_groups
// groups in all, none smaller than min_rows_per_group unless its build is; and, when the item
// table has room, no group larger than one chunk, so that no group merges through atomics.
__host__ __device__ inline int64_t hist_target_rows(const HistPlan& p, int64_t total, int n_entries) {
    int64_t t = (total + p.max_groups - 1) / p.max_groups;
    if (t < p.min_rows_per_group) t = p.min_rows_per_group;
    if (t > p.single_rows) {
        const int64_t room = (int64_t)p.max_items - n_entries - 1;
        if (total / p.single_rows < room) t = p.single_rows;
        else if (room > 0 && (total + room - 1) / room > t) t = (total + room - 1) / room;
    }
    return t;
}

struct ScanItem;

// Where the rows of a slice live.  Buffers 0..2 rotate with the depth of a node (the children
// of buffer b live in buffer (b+1)%3, so a node's rows survive until its grandchildren are
// expanded); buffer 3 is the caller's data in original row order (bin matrix, quantized
// gradients), where the root lives in ordered mode.  Row ids of buffer 3 use array 0.
// In ordered mode (narrow rows) buffers 0..2 hold leaf-ordered copies of the bin rows and
// packed gradients.  Otherwise the bin rows are gathered from the original matrix by row id;
// with `gh_pos` set the packed gradients still travel with the row ids (gh[b][p] belongs to
// row idx[b][p]: 2 more bytes per moved row, and a gathered build reads them in sequence
// instead of one more cache line per row), without it they are gathered from gh[BUF_ORIGINAL].
constexpr int BUF_ORIGINAL = 3;
struct RowSource {
    const uint8_t* bins[4];
    const int16_t* gh[4];
    int32_t gh_pos;
};
struct RowDest {
    uint8_t* bins[3];
    int16_t* gh[3];
};
struct IdxSet {
    int32_t* p[4];  // p[3] == p[0]
};
__host__ __device__ inline int child_buffer(int buf) { return buf == BUF_ORIGINAL ? 1 : (buf + 1) % 3; }

}  // namespace qgbdt

struct qgbdt_ctx {
    qgbdt_shape shape;
    hipStream_t stream;
    int device;
    // the caller's workspace block (qgbdt_set_workspace); every device pointer below points into it
    void* ws_base;
    size_t ws_bytes;
    uint32_t ws_flags;
    // sizes derived from the shape
    int batch_max;   // most nodes expanded per round
    int max_expand;  // most expansions per tree (sequential ones plus speculative ones)
    int max_nodes;
    int max_seg;
    int rounds_hint;
    // workspace
    int ordered;           // the workspace holds leaf-ordered copies of the rows (narrow rows, QGBDT_WS_ROW_COPIES)
    uint8_t* obins[3];     // [N][F] each (ordered mode), else null
    int16_t* ogh[3];       // [N] each: packed gradients in the order of idx[b]
    int32_t* idx[3];       // [N] each
    uint8_t* bins_t;       // [F][N] feature-major copy of the bound bin matrix (QGBDT_WS_BIND, filled by qgbdt_bind_bins), else null
    uint16_t* mfb;         // [F] most frequent bin of each feature of the bound matrix when it holds most rows, else 0xffff
    int mfb_features;      // features with such a bin (0: no skipping)
    const void* bound_bins; // the matrix that copy was made from
    int16_t* gh;           // [N]
    float2* ghf;           // [N] (g, h) interleaved, written by the quantizer for the refit's gather
    float* gbuf;           // [N] loss derivatives of a boosting iteration run by the library (QGBDT_WS_BOOST), else null
    float* hbuf;           // [N]
    int64_t* hist_pool;    // [max_expand + 1][nb*F]
    void* hist_partials;   // [max_items][n_tiles] local bins of the row groups, summed by the reduce kernel
    size_t hist_partials_bytes;
    uint8_t* flags;        // [N] partition flags
    int64_t* part_counts;  // [PART_GROUPS] (stand-alone partition)
    int32_t* seg_counts;   // [max_seg] left rows per partition segment
    int32_t* seg_prefix;   // [max_seg + 1]
    float* absmax_part;    // [QUANT_PARTS][2] per-workgroup max|g|, max h
    int64_t* qtotals_part; // [QUANT_PARTS][3] per-workgroup quantized totals
    int64_t* qtotals;      // [3] sum g~, sum h~, sum |g~|
    float* delta;          // [2]
    qgbdt::Node* nodes;          // [max_nodes]
    int32_t* sorted_idx;         // [max_nodes] node ids by descending gain, kept from round to round
    qgbdt::StepState* step;      // [1]
    qgbdt::BatchEntry* batch;    // [batch_max]
    qgbdt::FeatCand* cand;       // [2*batch_max][F]
    qgbdt::HistEntry* hist_entries;  // [batch_max]
    int32_t* hist_counts;        // [2] entries, items
    qgbdt::PartWork* pwork;      // [1]
    qgbdt::ScanItem* scan_items; // [2*batch_max]
    int32_t* leaf_node;          // [max_leaves]
    double* refit_partial;       // [max_leaves][REFIT_PARTS][2]
    int64_t* tmp_i64;            // [8]
    qgbdt::StepState* host_state;  // pinned host copy
    // profiling
    int profiling;
    hipEvent_t* ev;
    int ev_cap, ev_used;
    unsigned char* ev_root;  // [ev_cap / 2] 1: the launch was a tree's root build (all rows, contiguous)
    int next_hist_is_root;
    void* static_scratch;  // this device's copy of the library's fixed scratch array (entry points that allocate nothing)
    char err[512];
};

namespace qgbdt {

constexpr int PART_GROUPS = 512;
constexpr int REFIT_PARTS = 32;
constexpr int QUANT_PARTS = 2048;  // most workgroups of the quantizer kernels
constexpr int PART_SEG = 1024;  // rows per partition segment of the batched partition
// Most nodes expanded in one round = most builds of a histogram launch (the leaf budget; the growth bookkeeping
// limits it to 658).  Kernels keep the first work item of every build / node in LDS and search there: a binary
// search through global memory costs a chain of dependent loads per work item.
constexpr int TABLE_MAX = 768;

int set_error(qgbdt_ctx* ctx, int code, const char* fmt, ...);

#define QG_HIP(ctx, expr)                                                                      \
    do {                                                                                       \
        hipError_t e__ = (expr);                                                               \
        if (e__ != hipSuccess)                                                                 \
            return qgbdt::set_error(ctx, QGBDT_E_HIP, "%s failed: %s (%s:%d)", #expr,          \
                                    hipGetErrorString(e__), __FILE__, __LINE__);               \
    } while (0)

// launchers (each defined next to its kernels)
int launch_quantize(qgbdt_ctx* ctx, const float* g, const float* h, int64_t n, int bits_g, int bits_h,
                    uint64_t seed, uint32_t iteration, int rounding, int16_t* gh, float* delta_out,
                    int64_t* totals_out, float2* pairs_out);
HistPlan make_hist_plan(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width, bool skew = false);
HistPlan make_hist_plan_for(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width, int64_t rows, bool skew = false,
                            bool stream_ok = false);  // stream_ok: contiguous rows of a 16-byte aligned matrix
int64_t max_rows_for_width(int bits_g, int bits_h, int w);
int launch_set_hist_table(qgbdt_ctx* ctx, const HistPlan& plan, int64_t begin, int64_t count);
int launch_hist(qgbdt_ctx* ctx, const HistPlan& plan, const RowSource& rows, const IdxSet& idx, bool use_idx,
                bool flat_ok, const HistEntry* entries, const int32_t* table_counts, int64_t* hist_base,
                int64_t grid_items, StepState* step, const uint16_t* mfb = nullptr);
int launch_fill_zero(qgbdt_ctx* ctx, int64_t* p, int64_t n_words);
int launch_subtract(qgbdt_ctx* ctx, const int64_t* parent, const int64_t* child, int64_t* out, int64_t n);
int launch_scan_items(qgbdt_ctx* ctx, int64_t* hist_base, const ScanItem* items, const int32_t* n_items, int max_items,
                      const float* delta, int min_data, double min_sum_hess, FeatCand* cand, const uint16_t* mfb = nullptr,
                      bool reduce = true);  // reduce = false: the caller's next kernel reduces the per-feature candidates
// stand-alone search in batches of `cap` histograms; scratch: items [cap], cand [cap][F], n_items [1]
int run_find_best_splits(qgbdt_ctx* ctx, const int64_t* hist, int n_hists, const qgbdt_leafstat* stats,
                         const float* delta, int min_data, double min_sum_hess, qgbdt_split* out, int cap,
                         ScanItem* items, FeatCand* cand, int32_t* n_items);
int launch_partition_work(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* buf0, int32_t* buf1, const PartWork* work,
                          int64_t* n_left_out, int64_t max_count);
int run_partition_rows(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* row_idx, int64_t begin, int64_t count,
                       int feature, int bin, int64_t* n_left_out);
int launch_batch_partition_count(qgbdt_ctx* ctx, const RowSource& rows, const uint8_t* bins_t, bool ordered);
int launch_transpose_bins(qgbdt_ctx* ctx, const void* bins, void* out);
int launch_frequent_bins(qgbdt_ctx* ctx, const void* bins_t, uint16_t* mfb);
int launch_fix_frequent_bins(qgbdt_ctx* ctx, int64_t* hist, const int64_t* totals, const uint16_t* mfb);
int require_workspace(qgbdt_ctx* ctx);   // QGBDT_E_WORKSPACE unless a workspace block is set
int prepare_hist_kernels(qgbdt_ctx* ctx);  // once per context: dynamic-LDS limits of the kernels that exceed the default
int prepare_tree_kernels(qgbdt_ctx* ctx);
int launch_batch_partition_scatter(qgbdt_ctx* ctx, const RowSource& rows, bool ordered);  // !ordered: row ids and, with rows.gh_pos, packed gradients
int launch_refit(qgbdt_ctx* ctx, const float* g, const float* h, const float2* pairs, const int32_t* row_idx,
                 const int64_t* leaf_begin, const int64_t* leaf_count, int n_leaves,
                 const int32_t* n_leaves_dev, double* value_out);
int launch_logistic_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n, float* g, float* h);
int launch_lambdarank_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n, int group,
                                float* g, float* h);
int launch_update_scores(qgbdt_ctx* ctx, float* score, const int32_t* row_idx, const int64_t* leaf_begin,
                         const int64_t* leaf_count, const double* leaf_value, int n_leaves,
                         const int32_t* n_leaves_dev, double lr);
int run_grow_tree(qgbdt_ctx* ctx, const uint8_t* bins, const float* g, const float* h,
                  const qgbdt_params* p, uint32_t iteration, const qgbdt_tree* out, int32_t* row_idx_out);

}  // namespace qgbdt
