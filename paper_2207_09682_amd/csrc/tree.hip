// Leaf-wise growth of one tree (greedy splitting of Sec. 3, best-first order of
// Sec. 7) driven entirely from the device: the host enqueues a fixed sequence of
// kernels per split and never reads anything back; split decisions, leaf
// bookkeeping and the arguments of the next kernels live in device memory.  Once
// the tree is finished the remaining kernels of the sequence return at once.
#include "split_device.h"

namespace qgbdt {

struct TreeOut {
    qgbdt_tree t;
    int32_t max_leaves;
};

__global__ __launch_bounds__(256) void tree_init_kernel(int32_t* idx0, int64_t N, StepState* step, LeafState* leaves,
                                                        const int64_t* qtotals, HistWork* hwork, PartWork* pwork,
                                                        ScanItem* items, int64_t* hist0, int64_t hist_words) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < N; i += stride) idx0[i] = (int32_t)i;
    for (int64_t i = t; i < hist_words; i += stride) hist0[i] = 0;
    if (t == 0) {
        step->done = 0; step->n_leaves = 1; step->leaf = 0; step->new_leaf = 1;
        step->pending = 1; step->pend_leaf[0] = 0; step->pend_leaf[1] = -1;
        step->hist_units = 0; step->n_left = 0;
        LeafState r;
        r.begin = 0; r.count = N; r.sum_g = qtotals[0]; r.sum_h = qtotals[1]; r.buf = 0; r.slot = 0;
        r.best.gain = 0.0; r.best.feature = -1; r.best.bin = -1;
        r.best.left_g = r.best.left_h = r.best.right_g = r.best.right_h = r.best.left_count = 0;
        leaves[0] = r;
        hwork->begin = 0; hwork->count = N; hwork->use_idx = 0; hwork->buf = 0; hwork->slot = 0;
        pwork->count = 0; pwork->zero_slot = -1;
        items[0].slot = 0; items[0].sub_parent = -1; items[0].sub_child = -1; items[0].valid = 1;
        items[0].stat.n_rows = N; items[0].stat.sum_g = r.sum_g; items[0].stat.sum_h = r.sum_h;
        items[1].valid = 0;
    }
}

// Finishes the previous step (per-feature candidates -> best split of the two new
// leaves), then picks the open leaf with the largest gain (ties: lowest id) and
// publishes the partition work of split number k.
__global__ __launch_bounds__(256) void tree_choose_kernel(StepState* step, LeafState* leaves, const FeatCand* cand,
                                                          const ScanItem* items, int F, int num_leaves, int k,
                                                          PartWork* pwork, HistWork* hwork, ScanItem* items_w,
                                                          TreeOut out) {
    if (step->done) return;
    const int tid = threadIdx.x;
    if (step->pending) {
        for (int c = 0; c < 2; ++c) {
            const int l = step->pend_leaf[c];
            if (l >= 0) reduce_features(cand + (int64_t)c * F, F, items[c].stat, &leaves[l].best, tid, blockDim.x);
        }
    }
    __syncthreads();
    const int n = step->n_leaves;
    double bg = 0.0;
    int bl = -1;
    for (int l = tid; l < n; l += blockDim.x) {
        const qgbdt_split s = leaves[l].best;
        if (s.feature >= 0 && s.gain > bg) { bg = s.gain; bl = l; }
    }
    for (int o = 32; o > 0; o >>= 1) {
        const double og = __shfl_xor(bg, o);
        const int ol = __shfl_xor(bl, o);
        if (ol >= 0 && (bl < 0 || og > bg || (og == bg && ol < bl))) { bg = og; bl = ol; }
    }
    __shared__ double sg[4];
    __shared__ int sl[4];
    if ((tid & 63) == 0) { sg[tid >> 6] = bg; sl[tid >> 6] = bl; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w)
            if (sl[w] >= 0 && (bl < 0 || sg[w] > bg || (sg[w] == bg && sl[w] < bl))) { bg = sg[w]; bl = sl[w]; }
        step->pending = 0;
        if (bl < 0 || n >= num_leaves) {
            step->done = 1;
            pwork->count = 0; pwork->zero_slot = -1;
            hwork->count = 0;
            items_w[0].valid = 0; items_w[1].valid = 0;
            return;
        }
        const LeafState P = leaves[bl];
        step->leaf = bl; step->new_leaf = n;
        step->feature = P.best.feature; step->bin = P.best.bin;
        step->src_buf = P.buf; step->begin = P.begin; step->count = P.count;
        step->parent_slot = P.slot; step->new_slot = n;
        pwork->begin = P.begin; pwork->count = P.count; pwork->feature = P.best.feature; pwork->bin = P.best.bin;
        pwork->src_buf = P.buf; pwork->zero_slot = n;
        out.t.split_leaf[k] = bl; out.t.split_feature[k] = P.best.feature; out.t.split_bin[k] = P.best.bin;
        out.t.split_gain[k] = P.best.gain;
        out.t.split_stats[4 * k + 0] = P.best.left_g; out.t.split_stats[4 * k + 1] = P.best.left_h;
        out.t.split_stats[4 * k + 2] = P.best.right_g; out.t.split_stats[4 * k + 3] = P.best.right_h;
    }
}

// After the partition: children's slices and totals, which child is built from its
// rows (fewer rows, tie: left) and which by subtraction, and the work of the
// histogram and scan kernels that follow.
__global__ void tree_after_partition_kernel(StepState* step, LeafState* leaves, HistWork* hwork, ScanItem* items,
                                            int k, TreeOut out) {
    if (threadIdx.x != 0 || step->done) return;
    const int s = step->leaf, r = step->new_leaf;
    const LeafState P = leaves[s];
    const int64_t nl = step->n_left, nr = step->count - nl;
    out.t.split_n_left[k] = nl;
    const int small_is_left = (nl <= nr) ? 1 : 0;
    step->small_is_left = small_is_left;
    const int child_buf = 1 - step->src_buf;
    LeafState L, R;
    L.begin = step->begin; L.count = nl; L.sum_g = P.best.left_g; L.sum_h = P.best.left_h; L.buf = child_buf;
    R.begin = step->begin + nl; R.count = nr; R.sum_g = P.best.right_g; R.sum_h = P.best.right_h; R.buf = child_buf;
    L.slot = small_is_left ? step->new_slot : step->parent_slot;
    R.slot = small_is_left ? step->parent_slot : step->new_slot;
    L.best.gain = 0.0; L.best.feature = -1; L.best.bin = -1;
    L.best.left_g = L.best.left_h = L.best.right_g = L.best.right_h = L.best.left_count = 0;
    R.best = L.best;
    leaves[s] = L; leaves[r] = R;
    const LeafState& S = small_is_left ? L : R;
    hwork->begin = S.begin; hwork->count = S.count; hwork->use_idx = 1; hwork->buf = child_buf;
    hwork->slot = step->new_slot;
    for (int c = 0; c < 2; ++c) {
        const LeafState& C = c ? R : L;
        const bool is_small = (c == 0) == (small_is_left == 1);
        items[c].slot = C.slot;
        items[c].sub_parent = is_small ? -1 : step->parent_slot;
        items[c].sub_child = is_small ? -1 : step->new_slot;
        items[c].valid = 1;
        items[c].stat.n_rows = C.count; items[c].stat.sum_g = C.sum_g; items[c].stat.sum_h = C.sum_h;
    }
    step->pend_leaf[0] = s; step->pend_leaf[1] = r; step->pending = 1;
    step->n_leaves = r + 1;
}

__global__ void tree_finalize_kernel(const StepState* step, const LeafState* leaves, const float* delta,
                                     TreeOut out) {
    const int n = step->n_leaves;
    const double dg = (double)delta[0], dh = (double)delta[1];
    for (int l = threadIdx.x; l < out.max_leaves; l += blockDim.x) {
        if (l < n) {
            const LeafState S = leaves[l];
            out.t.leaf_begin[l] = S.begin; out.t.leaf_count[l] = S.count;
            out.t.leaf_sum_g[l] = S.sum_g; out.t.leaf_sum_h[l] = S.sum_h;
            out.t.leaf_value_quant[l] =
                (S.sum_h > 0 && dh > 0.0) ? -((double)S.sum_g * dg) / ((double)S.sum_h * dh) : 0.0;
        } else {
            out.t.leaf_begin[l] = 0; out.t.leaf_count[l] = 0; out.t.leaf_sum_g[l] = 0; out.t.leaf_sum_h[l] = 0;
            out.t.leaf_value_quant[l] = 0.0;
        }
    }
    if (threadIdx.x == 0) {
        *out.t.n_leaves = n;
        out.t.delta[0] = delta[0]; out.t.delta[1] = delta[1];
        *out.t.hist_units = step->hist_units;
    }
}

// Copies every leaf's slice from the index buffer it ended up in to the output.
__global__ __launch_bounds__(256) void tree_gather_rows_kernel(const StepState* step, const LeafState* leaves,
                                                               const int32_t* __restrict__ idx0,
                                                               const int32_t* __restrict__ idx1,
                                                               int32_t* __restrict__ out) {
    const int l = blockIdx.y;
    if (l >= step->n_leaves) return;
    const LeafState S = leaves[l];
    const int32_t* src = S.buf ? idx1 : idx0;
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < S.count; j += (int64_t)gridDim.x * blockDim.x)
        out[S.begin + j] = src[S.begin + j];
}

int run_grow_tree(qgbdt_ctx* ctx, const uint8_t* bins, const float* g, const float* h, const qgbdt_params* p,
                  uint32_t iteration, const qgbdt_tree* tout, int32_t* row_idx_out) {
    const int64_t N = ctx->shape.n_rows;
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    const int64_t W = (int64_t)F * nb;
    ScanItem* items = reinterpret_cast<ScanItem*>(ctx->scan_items);
    TreeOut out;
    out.t = *tout;
    out.max_leaves = ctx->shape.max_leaves;

    int rc = launch_quantize(ctx, g, h, N, p->bits_g, p->bits_h, p->seed, iteration, p->rounding, ctx->gh,
                             ctx->delta, ctx->qtotals);
    if (rc != QGBDT_OK) return rc;
    // 32|32 words of the total histograms must hold the root's sums
    if (N > max_rows_for_width(p->bits_g, p->bits_h, 32)) {
        int64_t tot[3];
        QG_HIP(ctx, hipMemcpyAsync(tot, ctx->qtotals, sizeof(tot), hipMemcpyDeviceToHost, ctx->stream));
        QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (tot[1] > 0xffffffffLL || tot[2] > 0x7fffffffLL)
            return set_error(ctx, QGBDT_E_OVERFLOW_RISK,
                             "quantized totals (sum h~ = %lld, sum |g~| = %lld) do not fit 32|32 packed bins",
                             (long long)tot[1], (long long)tot[2]);
    }
    const HistPlan plan = make_hist_plan(ctx->shape, p->bits_g, p->bits_h, p->acc_width);

    int blocks = (int)((N + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(tree_init_kernel, dim3(blocks), dim3(256), 0, ctx->stream, ctx->idx[0], N, ctx->step,
                       ctx->leaves, ctx->qtotals, ctx->hwork, ctx->pwork, items, ctx->hist_pool, W);
    rc = launch_hist(ctx, plan, bins, ctx->gh, ctx->idx[0], ctx->idx[1], ctx->hwork, ctx->hist_pool, N, ctx->step);
    if (rc != QGBDT_OK) return rc;
    rc = launch_scan_items(ctx, ctx->hist_pool, items, 2, ctx->delta, p->min_data_in_leaf, p->min_sum_hessian,
                           ctx->cand);
    if (rc != QGBDT_OK) return rc;

    for (int k = 0; k + 1 < p->num_leaves; ++k) {
        hipLaunchKernelGGL(tree_choose_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->step, ctx->leaves, ctx->cand,
                           items, F, p->num_leaves, k, ctx->pwork, ctx->hwork, items, out);
        rc = launch_partition_work(ctx, bins, ctx->idx[0], ctx->idx[1], ctx->pwork, &ctx->step->n_left, N);
        if (rc != QGBDT_OK) return rc;
        hipLaunchKernelGGL(tree_after_partition_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->step, ctx->leaves,
                           ctx->hwork, items, k, out);
        rc = launch_hist(ctx, plan, bins, ctx->gh, ctx->idx[0], ctx->idx[1], ctx->hwork, ctx->hist_pool, N / 2 + 1,
                         ctx->step);
        if (rc != QGBDT_OK) return rc;
        rc = launch_scan_items(ctx, ctx->hist_pool, items, 2, ctx->delta, p->min_data_in_leaf, p->min_sum_hessian,
                               ctx->cand);
        if (rc != QGBDT_OK) return rc;
    }
    hipLaunchKernelGGL(tree_finalize_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->step, ctx->leaves, ctx->delta,
                       out);
    int gx = (int)((N / ctx->shape.max_leaves + 255) / 256);
    if (gx < 1) gx = 1;
    if (gx > 64) gx = 64;
    hipLaunchKernelGGL(tree_gather_rows_kernel, dim3(gx, ctx->shape.max_leaves), dim3(256), 0, ctx->stream, ctx->step,
                       ctx->leaves, ctx->idx[0], ctx->idx[1], row_idx_out);
    QG_HIP(ctx, hipGetLastError());
    return launch_refit(ctx, g, h, row_idx_out, out.t.leaf_begin, out.t.leaf_count, ctx->shape.max_leaves,
                        out.t.n_leaves, out.t.leaf_value);
}

}  // namespace qgbdt
