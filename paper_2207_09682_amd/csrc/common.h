// Internal declarations shared by the HIP translation units of libqgbdt.
// Nothing here is part of the public boundary (see include/qgbdt.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/qgbdt.h"

namespace qgbdt {

// ---- device-side bookkeeping of one tree -----------------------------------

// Per-leaf record kept on the device while a tree grows.
struct LeafState {
    int64_t begin, count;  // slice of the index buffer `buf`
    int64_t sum_g, sum_h;  // quantized totals
    int32_t buf;           // which of the two index buffers holds the slice
    int32_t slot;          // histogram slot in the pool
    qgbdt_split best;      // best split of this leaf (feature < 0: none)
};

// Work of the current split step; written by one kernel, read by the next ones.
struct StepState {
    int32_t done;        // 1: tree finished, later kernels return at once
    int32_t n_leaves;    // leaves so far
    int32_t leaf;        // leaf being split (left child keeps this id)
    int32_t new_leaf;    // id of the right child
    int32_t feature, bin;
    int32_t src_buf;     // index buffer holding the parent's slice
    int32_t small_is_left;
    int64_t begin, count;  // parent's slice
    int64_t n_left;        // true left count (after partition)
    int32_t parent_slot, new_slot;
    int32_t pending;       // 1: pend_leaf[] still need their per-feature candidates reduced
    int32_t pend_leaf[2];  // leaves whose candidates sit in the candidate buffer (-1: none)
    int32_t pad;
    int64_t hist_units;    // sum of rows*features accumulated by histogram builds
    int64_t prof_rows_contig, prof_rows_idx;  // rows seen by histogram launches
    int64_t prof_launches;                    // histogram launches that had rows
};

// Candidate of one (leaf, feature) pair produced by the scan kernel.
struct FeatCand {
    double gain;
    int64_t left;  // packed prefix word (G_L | H_L)
    int32_t bin;   // -1: no valid candidate
    int32_t pad;
};

// Work descriptor of one row partition.
struct PartWork {
    int64_t begin, count;
    int32_t feature, bin;
    int32_t src_buf;    // which index buffer holds the slice; the result goes to the other one
    int32_t zero_slot;  // >= 0: histogram slot cleared on the way (grow_tree)
};

// Work descriptor of one histogram build.
struct HistWork {
    int64_t begin, count;
    int32_t use_idx;  // rows come from an index buffer
    int32_t buf;      // which index buffer (grow_tree) -- 0 for the standalone call
    int32_t slot;     // histogram slot (grow_tree)
    int32_t pad;
};

struct HistPlan {
    int32_t ft;          // features per workgroup tile (multiple of 4)
    int32_t ftp;         // padded tile width in LDS words
    int32_t dpr;         // dwords per row per tile = ft/4
    int32_t rows_per_it; // rows one wavefront covers per iteration
    int32_t n_tiles;     // feature tiles
    int32_t threads;     // workgroup size
    int32_t lds_bytes;
    int32_t chunk_rows;  // rows accumulated between two merges of the local bins
    int32_t max_groups;  // workgroups along the row axis
    int32_t min_rows_per_group;
    int32_t acc_width;   // 16: packed 16|16 words in LDS, 32: packed 32|32 words
};

}  // namespace qgbdt

struct qgbdt_ctx {
    qgbdt_shape shape;
    hipStream_t stream;
    int device;
    size_t ws_bytes;
    // workspace
    int32_t* idx[2];       // [N] each
    int16_t* gh;           // [N]
    int64_t* hist_pool;    // [max_leaves][F*nb]
    uint8_t* flags;        // [N] partition flags
    int64_t* part_counts;  // [PART_GROUPS]
    uint32_t* absmax;      // [2] float bits
    int64_t* qtotals;      // [3] sum g~, sum h~, sum |g~|
    float* delta;          // [2]
    qgbdt::LeafState* leaves;  // [max_leaves]
    qgbdt::StepState* step;    // [1]
    qgbdt::FeatCand* cand;     // [2][F]
    qgbdt::HistWork* hwork;    // [1]
    qgbdt::PartWork* pwork;    // [1]
    void* scan_items;          // ScanItem[2]
    qgbdt_leafstat* tmp_stats; // [2]
    double* refit_partial;     // [max_leaves][REFIT_PARTS][2]
    int64_t* tmp_i64;          // [8]
    // profiling
    int profiling;
    hipEvent_t* ev;
    int ev_cap, ev_used;
    int64_t prof_launches;
    char err[512];
};

namespace qgbdt {

constexpr int PART_GROUPS = 512;
constexpr int REFIT_PARTS = 32;

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
                    int64_t* totals_out);
HistPlan make_hist_plan(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width);
int64_t max_rows_for_width(int bits_g, int bits_h, int w);
int launch_hist(qgbdt_ctx* ctx, const HistPlan& plan, const uint8_t* bins, const int16_t* gh,
                const int32_t* idx0, const int32_t* idx1, const HistWork* work, int64_t* hist_base,
                int64_t max_count, StepState* step);
int launch_fill_zero(qgbdt_ctx* ctx, int64_t* p, int64_t n_words);
int launch_subtract(qgbdt_ctx* ctx, const int64_t* parent, const int64_t* child, int64_t* out, int64_t n);
struct ScanItem;
int launch_scan_items(qgbdt_ctx* ctx, int64_t* hist_base, const ScanItem* items, int n_items, const float* delta,
                      int min_data, double min_sum_hess, FeatCand* cand);
int run_find_best_splits(qgbdt_ctx* ctx, const int64_t* hist, int n_hists, const qgbdt_leafstat* stats,
                         const float* delta, int min_data, double min_sum_hess, qgbdt_split* out);
int launch_partition_work(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* buf0, int32_t* buf1, const PartWork* work,
                          int64_t* n_left_out, int64_t max_count);
int run_partition_rows(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* row_idx, int64_t begin, int64_t count,
                       int feature, int bin, int64_t* n_left_out);
int launch_refit(qgbdt_ctx* ctx, const float* g, const float* h, const int32_t* row_idx,
                 const int64_t* leaf_begin, const int64_t* leaf_count, int n_leaves,
                 const int32_t* n_leaves_dev, double* value_out);
int run_grow_tree(qgbdt_ctx* ctx, const uint8_t* bins, const float* g, const float* h,
                  const qgbdt_params* p, uint32_t iteration, const qgbdt_tree* out, int32_t* row_idx_out);

}  // namespace qgbdt
