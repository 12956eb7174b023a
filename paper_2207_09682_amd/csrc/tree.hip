// Leaf-wise growth of one tree (greedy splitting of Sec. 3, best-first order of
// Sec. 7), driven from the device.
//
// Best-first growth is sequential by definition: split the open leaf with the
// largest gain, look at its children, repeat.  Its result, however, only depends on
// the gains, so it can be reproduced exactly from a tree that was expanded in a
// different order.  The tree is therefore grown in rounds.  Each round
//   1. replays the best-first order over what is known (commit phase): the open leaf
//      with the largest gain is committed as the next split if it has already been
//      expanded, and its children become open leaves; the replay stops at the first
//      leaf that has not been expanded;
//   2. expands that leaf and, speculatively, the other open leaves with the largest
//      gains (as many as the leaf budget still allows): one batched partition, one
//      batched histogram build for the smaller children, one batched subtraction and
//      split search for all children.
// A speculative expansion that the replay never reaches is simply not part of the
// tree: its node stays a leaf and its row slice is untouched, because children are
// always written to the other index buffer.  Split numbers and leaf ids are assigned
// at commit time, so the result equals the sequential one bit for bit.
//
// The host enqueues whole rounds without reading anything back; after the expected
// number of rounds it reads one status word to learn whether more are needed.
#include "split_device.h"

namespace qgbdt {

struct TreeOut {
    qgbdt_tree t;
    int32_t max_leaves;
};

__device__ __forceinline__ void clear_split(qgbdt_split& s) {
    s.gain = 0.0; s.feature = -1; s.bin = -1;
    s.left_g = s.left_h = s.right_g = s.right_h = s.left_count = 0;
}

__device__ __forceinline__ int hist_groups(int64_t count, const HistPlan& plan) {
    const int64_t t = hist_target_rows(plan, count, 1);
    int64_t g = (count + t - 1) / t;
    if (g < 1) g = 1;
    return (int)g;
}

__global__ __launch_bounds__(256) void tree_init_kernel(int32_t* idx0, int64_t N, int F, StepState* step, Node* nodes,
                                                        const int64_t* qtotals, int root_buf, HistEntry* hist_entries,
                                                        int32_t* hist_counts, ScanItem* items, int32_t* scan_counters,
                                                        int64_t* hist0, int64_t hist_words, HistPlan plan) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < N; i += stride) idx0[i] = (int32_t)i;
    for (int64_t i = t; i < hist_words; i += stride) hist0[i] = 0;
    if (t == 0) {
        step->done = 0; step->n_nodes = 1; step->n_leaves = 1; step->n_commits = 0; step->n_expanded = 0;
        step->n_slots = 1; step->n_batch = 0; step->rounds = 0; step->n_part_items = 0; step->n_scan_items = 1;
        step->hist_units = N * (int64_t)F;
        Node r;
        r.begin = 0; r.count = N; r.sum_g = qtotals[0]; r.sum_h = qtotals[1]; r.n_left = 0; r.buf = root_buf; r.slot = 0;
        r.state = 1; r.expanded = 0; r.child = -1; r.leaf_id = 0;
        clear_split(r.best);
        nodes[0] = r;
        HistEntry e;
        e.begin = 0; e.count = N; e.buf = root_buf; e.slot = 0; e.item_start = 0; e.groups = hist_groups(N, plan);
        hist_entries[0] = e;
        hist_counts[0] = 1; hist_counts[1] = e.groups;
        ScanItem it;
        it.slot = 0; it.sub_parent = -1; it.sub_child = -1; it.valid = 1;
        it.stat.n_rows = N; it.stat.sum_g = r.sum_g; it.stat.sum_h = r.sum_h;
        it.out = &nodes[0].best;
        items[0] = it;
        scan_counters[0] = 0;
    }
}

// Inclusive scan of one int per thread over the workgroup (1024 threads).
__device__ __forceinline__ int block_scan_incl(int v, int* tmp /*[16]*/) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int o = 1; o < 64; o <<= 1) {
        const int u = __shfl_up(v, o);
        if (lane >= o) v += u;
    }
    __syncthreads();
    if (lane == 63) tmp[wave] = v;
    __syncthreads();
    int add = 0;
    for (int k = 0; k < wave; ++k) add += tmp[k];
    return v + add;
}

// Wavefront-wide maximum of one unsigned value per lane with DPP moves (no LDS traffic);
// the result is uniform.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
#define QG_DPP(x, ctrl, rmask) (uint32_t)__builtin_amdgcn_update_dpp((int)(x), (int)(x), ctrl, rmask, 0xf, false)
    v = max(v, QG_DPP(v, 0xB1, 0xf));   // quad_perm [1,0,3,2]
    v = max(v, QG_DPP(v, 0x4E, 0xf));   // quad_perm [2,3,0,1]
    v = max(v, QG_DPP(v, 0x141, 0xf));  // row_half_mirror
    v = max(v, QG_DPP(v, 0x140, 0xf));  // row_mirror: every lane of a row holds the row's maximum
    v = max(v, QG_DPP(v, 0x142, 0xa));  // row_bcast:15 into rows 1 and 3
    v = max(v, QG_DPP(v, 0x143, 0xc));  // row_bcast:31 into rows 2 and 3
#undef QG_DPP
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Commit phase and choice of the round's batch.  One workgroup of 1024 threads; the
// replay itself runs in its first wavefront on an LDS copy of the queue (gain, leaf id,
// children, expanded flag of every node) and only records the order of the commits; the
// outputs of the committed splits are then written by all threads.
__global__ __launch_bounds__(1024) void tree_plan_kernel(StepState* step, Node* nodes, BatchEntry* batch,
                                                         int32_t* hist_counts, int32_t* scan_counters, int F,
                                                         int num_leaves, int batch_max, int max_expand, TreeOut out) {
    if (step->done) return;
    extern __shared__ unsigned char plan_lds[];
    const int n_nodes0 = step->n_nodes;
    const int cap = 2 * max_expand + 1;                 // nodes
    double* key = reinterpret_cast<double*>(plan_lds);  // gain of the node's best split, -1 if it has none
    int* lid = reinterpret_cast<int*>(key + cap);       // leaf id (open leaves)
    int* child = lid + cap;                             // left child, -1 if not expanded
    // open leaves that can be split: unordered list of (node, gain bits, leaf id), [num_leaves+1] each
    int* o_node = child + cap;
    uint32_t* o_hi = reinterpret_cast<uint32_t*>(o_node + num_leaves + 1);
    uint32_t* o_lo = o_hi + num_leaves + 1;
    uint32_t* o_lid = o_lo + num_leaves + 1;
    int* commit = reinterpret_cast<int*>(o_lid + num_leaves + 1);  // [num_leaves] nodes committed in this call, in order
    int* cand = commit + num_leaves + 1;                           // [3*num_leaves] candidates of the batch selection
    __shared__ int s_tmp[16];
    __shared__ int s_done, s_ncand, s_nopen, s_ncommit, s_commits0, s_leaves0;
    __shared__ unsigned long long s_units;
    const int tid = threadIdx.x;
    if (tid == 0) { s_done = 0; s_ncand = 0; s_nopen = 0; s_ncommit = 0; s_units = 0ull; }
    __syncthreads();
    for (int i = tid; i < n_nodes0; i += blockDim.x) {
        const Node* nd = &nodes[i];
        const double kg = (nd->best.feature >= 0 && nd->state != 2) ? nd->best.gain : -1.0;
        key[i] = kg;
        lid[i] = nd->leaf_id;
        child[i] = nd->expanded ? nd->child : -1;
        if (nd->state == 1 && kg > 0.0) {
            const int p = atomicAdd(&s_nopen, 1);
            o_node[p] = i; o_hi[p] = (uint32_t)__double2hiint(kg); o_lo[p] = (uint32_t)__double2loint(kg);
            o_lid[p] = (uint32_t)nd->leaf_id;
        }
    }
    __syncthreads();

    if (tid < 64) {
        // Replay of the best-first order by one wavefront, LDS and registers only.  A positive
        // double orders like its bit pattern, so the largest gain (ties: lowest leaf id) is found
        // by three wavefront-wide maxima: high word, low word among the high word's winners,
        // complemented leaf id among those.
        const int commits0 = step->n_commits, leaves0 = step->n_leaves;
        int n_commits = commits0, n_leaves = leaves0, n_open = s_nopen;
        for (;;) {
            if (n_commits >= num_leaves - 1) { if (tid == 0) s_done = 1; break; }
            if (n_open <= 0) { if (tid == 0) s_done = 1; break; }  // no open leaf has a gain > 0
            uint32_t bh = 0, bl = 0, bd = 0xffffffffu;
            int bp = -1;
            for (int p = tid; p < n_open; p += 64) {
                const uint32_t h = o_hi[p], l = o_lo[p], d = o_lid[p];
                if (bp < 0 || h > bh || (h == bh && (l > bl || (l == bl && d < bd)))) { bh = h; bl = l; bd = d; bp = p; }
            }
            const uint32_t mh = wave_max_u32(bp >= 0 ? bh : 0u);
            const bool in1 = bp >= 0 && bh == mh;
            const uint32_t ml = wave_max_u32(in1 ? bl : 0u);
            const bool in2 = in1 && bl == ml;
            const uint32_t md = ~wave_max_u32(in2 ? ~bd : 0u);
            const unsigned long long win = __ballot(in2 && bd == md);
            const int wl = __ffsll((long long)win) - 1;
            const int wp = __builtin_amdgcn_readlane(bp, wl);
            const int bi = o_node[wp];
            const int c0 = child[bi];
            if (c0 < 0) break;  // the next split is not known yet
            // commit: the node leaves the queue, its children enter (left keeps the leaf id)
            const double k0 = key[c0], k1 = key[c0 + 1];
            const int add0 = k0 > 0.0, add1 = k1 > 0.0;
            if (tid == 0) {
                commit[n_commits - commits0] = bi;
                key[bi] = -1.0;
                lid[c0] = (int)md; lid[c0 + 1] = n_leaves;
                const int last = n_open - 1;
                o_node[wp] = o_node[last]; o_hi[wp] = o_hi[last]; o_lo[wp] = o_lo[last]; o_lid[wp] = o_lid[last];
                int no = last;
                if (add0) {
                    o_node[no] = c0; o_hi[no] = (uint32_t)__double2hiint(k0); o_lo[no] = (uint32_t)__double2loint(k0);
                    o_lid[no] = md; ++no;
                }
                if (add1) {
                    o_node[no] = c0 + 1; o_hi[no] = (uint32_t)__double2hiint(k1); o_lo[no] = (uint32_t)__double2loint(k1);
                    o_lid[no] = (uint32_t)n_leaves; ++no;
                }
            }
            n_open += add0 + add1 - 1;
            n_commits += 1; n_leaves += 1;
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
        if (tid == 0) {
            s_ncommit = n_commits - commits0; s_commits0 = commits0; s_leaves0 = leaves0; s_nopen = n_open;
            step->n_commits = n_commits; step->n_leaves = n_leaves;
        }
    }
    __syncthreads();
    // outputs and node states of the splits committed above
    for (int c = tid; c < s_ncommit; c += blockDim.x) {
        const int i = commit[c], k = s_commits0 + c;
        const Node nd = nodes[i];
        out.t.split_leaf[k] = lid[i]; out.t.split_feature[k] = nd.best.feature; out.t.split_bin[k] = nd.best.bin;
        out.t.split_gain[k] = nd.best.gain;
        out.t.split_stats[4 * k + 0] = nd.best.left_g; out.t.split_stats[4 * k + 1] = nd.best.left_h;
        out.t.split_stats[4 * k + 2] = nd.best.right_g; out.t.split_stats[4 * k + 3] = nd.best.right_h;
        out.t.split_n_left[k] = nd.n_left;
        const int64_t nl = nd.n_left, nr = nd.count - nd.n_left;
        atomicAdd(&s_units, (unsigned long long)((nl <= nr ? nl : nr) * (int64_t)F));
        nodes[nd.child].state = 1; nodes[nd.child].leaf_id = lid[nd.child];
        nodes[nd.child + 1].state = 1; nodes[nd.child + 1].leaf_id = lid[nd.child + 1];
    }
    __syncthreads();  // a child may itself have been committed in this call: "internal" is written last
    for (int c = tid; c < s_ncommit; c += blockDim.x) nodes[commit[c]].state = 2;
    if (tid == 0) step->hist_units += (int64_t)s_units;
    __syncthreads();
    if (s_done) {
        if (tid == 0) {
            step->done = 1; step->n_batch = 0; step->n_part_items = 0; step->n_scan_items = 0;
            hist_counts[0] = 0; hist_counts[1] = 0;
        }
        return;
    }
    // batch: the open, not yet expanded leaves with the largest gains.  One expansion is
    // certain (the leaf the replay stopped at); slots beyond those that the remaining certain
    // expansions will need may be spent on speculation.
    const int remaining = (num_leaves - 1) - step->n_commits;
    const int spare = (max_expand - step->n_expanded) - remaining;
    int want = 1 + (spare > 0 ? spare : 0);
    if (want > remaining) want = remaining;
    if (want > batch_max) want = batch_max;
    // Candidates: open leaves that are not expanded yet (class 0: the leaf the replay stopped at is
    // the best of them) and, one level ahead, the not yet expanded children of expanded open leaves
    // (class 1; encoded as -1-node).  A node's rows outlive the expansion of its children, so
    // expanding the children of a leaf whose split is not committed yet is safe.
    for (int p = tid; p < s_nopen; p += blockDim.x) {
        const int i = o_node[p];
        const int c0 = child[i];
        if (c0 < 0) {
            cand[atomicAdd(&s_ncand, 1)] = i;
        } else {
            if (key[c0] > 0.0 && child[c0] < 0) cand[atomicAdd(&s_ncand, 1)] = -1 - c0;
            if (key[c0 + 1] > 0.0 && child[c0 + 1] < 0) cand[atomicAdd(&s_ncand, 1)] = -1 - (c0 + 1);
        }
    }
    __syncthreads();
    const int nc = s_ncand;
    // Rank of every candidate's gain among all nodes that may still be committed (every known,
    // not committed node with a gain > 0; ties by node id).  A candidate that already has
    // `remaining` better nodes in front of it is not worth expanding yet.  Four threads share
    // one candidate's pass over the nodes.
    int* crank = cand + 3 * num_leaves;  // [3*num_leaves]
    for (int c = tid; c < nc; c += blockDim.x) crank[c] = 0;
    __syncthreads();
    for (int w = tid; w < 4 * nc; w += blockDim.x) {
        const int c = w >> 2, part = w & 3;
        const int e = cand[c];
        const int i = e < 0 ? -1 - e : e;
        const double g = key[i];
        int r = 0;
        for (int j = part; j < n_nodes0; j += 4) {
            const double go = key[j];
            r += (go > g || (go == g && j < i)) ? 1 : 0;
        }
        atomicAdd(&crank[c], r);
    }
    __syncthreads();
    // order of the batch: class 0 first, then class 1, each by rank; the best class-0 candidate
    // (the leaf the replay stopped at) always passes the filter
    int* posbuf = crank + 3 * num_leaves;  // [3*num_leaves + 2] node per position, -1 = filtered out
    for (int c = tid; c < nc; c += blockDim.x) {
        const int e = cand[c];
        const int cls = e < 0 ? 1 : 0;
        const int rk = crank[c];
        int pos = 0, better0 = 0;
        for (int j = 0; j < nc; ++j) {
            const int cj = cand[j] < 0 ? 1 : 0, rj = crank[j];
            pos += ((cj < cls) || (cj == cls && rj < rk)) ? 1 : 0;
            better0 += (cj == 0 && rj < rk) ? 1 : 0;
        }
        const bool pass = (cls == 0 && better0 == 0) || rk < remaining;
        posbuf[pos] = pass ? (e < 0 ? -1 - e : e) : -1;
    }
    __syncthreads();
    // compaction of the passing candidates in position order (two positions per thread)
    const int p0 = 2 * tid, p1 = 2 * tid + 1;
    const int f0 = (p0 < nc && posbuf[p0] >= 0) ? 1 : 0, f1 = (p1 < nc && posbuf[p1] >= 0) ? 1 : 0;
    const int pincl = block_scan_incl(f0 + f1, s_tmp);
    __shared__ int s_npass;
    if (tid == (int)blockDim.x - 1) s_npass = pincl;
    __syncthreads();
    const int n_pass = s_npass;
    const int n_batch = n_pass < want ? n_pass : want;
    {
        int o = pincl - (f0 + f1);
        if (f0) { if (o < n_batch) batch[o].node = posbuf[p0]; ++o; }
        if (f1) { if (o < n_batch) batch[o].node = posbuf[p1]; }
    }
    __syncthreads();
    __threadfence_block();
    // segments of the batched partition, new histogram slots, child ids
    int nseg = 0;
    if (tid < n_batch) nseg = (int)((nodes[batch[tid].node].count + PART_SEG - 1) / PART_SEG);
    const int incl = block_scan_incl(nseg, s_tmp);
    const int n_nodes = n_nodes0, n_slots = step->n_slots;
    if (tid < n_batch) {
        const int i = batch[tid].node;
        batch[tid].seg_start = incl - nseg;
        batch[tid].n_seg = nseg;
        batch[tid].new_slot = n_slots + tid;
        nodes[i].expanded = 1;
        nodes[i].child = n_nodes + 2 * tid;
        scan_counters[2 * tid] = 0; scan_counters[2 * tid + 1] = 0;
    }
    if (tid == n_batch - 1) step->n_part_items = incl;
    {   // diagnostics: rows partitioned in this round
        int rows_k = 0;
        if (tid < n_batch) rows_k = (int)((nodes[batch[tid].node].count + 1023) >> 10);
        const int tot = block_scan_incl(rows_k, s_tmp);
        if (tid == (int)blockDim.x - 1 && step->rounds < 96) { step->round_rows[step->rounds] = (int64_t)tot << 10; step->round_batch[step->rounds] = n_batch; }
    }
    __syncthreads();
    if (tid == 0) {
        step->n_batch = n_batch;
        step->n_nodes = n_nodes + 2 * n_batch;
        step->n_slots = n_slots + n_batch;
        step->n_expanded += n_batch;
        step->rounds += 1;
        step->n_scan_items = 2 * n_batch;
    }
}

// Between the two partition passes: exclusive prefix of the segments' left counts, the
// children of every expanded node, and the tables of the histogram and scan kernels.
__global__ __launch_bounds__(1024) void tree_mid_kernel(StepState* step, Node* nodes, const BatchEntry* batch,
                                                        const int32_t* seg_counts, int32_t* seg_prefix,
                                                        HistEntry* hist_entries, int32_t* hist_counts, ScanItem* items,
                                                        HistPlan plan) {
    if (step->done) return;
    __shared__ int s_tmp[16];
    const int tid = threadIdx.x;
    const int n_items = step->n_part_items, n_batch = step->n_batch;
    // prefix over all segments: every thread owns a contiguous run
    const int per = (n_items + blockDim.x - 1) / blockDim.x;
    const int a = min(tid * per, n_items), b = min(a + per, n_items);
    int local = 0;
    for (int i = a; i < b; ++i) local += seg_counts[i];
    const int incl = block_scan_incl(local, s_tmp);
    int run = incl - local;
    for (int i = a; i < b; ++i) { seg_prefix[i] = run; run += seg_counts[i]; }
    if (tid == (int)blockDim.x - 1) seg_prefix[n_items] = incl;
    __syncthreads();
    __threadfence_block();
    int groups = 0, small_rows = 0;
    Node L, R;
    int small_is_left = 1;
    if (tid < n_batch) {
        const BatchEntry be = batch[tid];
        const Node P = nodes[be.node];
        const int64_t nl = seg_prefix[be.seg_start + be.n_seg] - seg_prefix[be.seg_start];
        const int64_t nr = P.count - nl;
        nodes[be.node].n_left = nl;
        small_is_left = (nl <= nr) ? 1 : 0;
        const int cb = child_buffer(P.buf);
        L.begin = P.begin; L.count = nl; L.sum_g = P.best.left_g; L.sum_h = P.best.left_h; L.n_left = 0; L.buf = cb;
        R.begin = P.begin + nl; R.count = nr; R.sum_g = P.best.right_g; R.sum_h = P.best.right_h; R.n_left = 0; R.buf = cb;
        L.slot = small_is_left ? be.new_slot : P.slot;
        R.slot = small_is_left ? P.slot : be.new_slot;
        L.state = 0; L.expanded = 0; L.child = -1; L.leaf_id = -1; clear_split(L.best);
        R.state = 0; R.expanded = 0; R.child = -1; R.leaf_id = -1; clear_split(R.best);
        nodes[P.child] = L; nodes[P.child + 1] = R;
        small_rows = (int)(small_is_left ? nl : nr);
        for (int c = 0; c < 2; ++c) {
            const Node& C = c ? R : L;
            const bool is_small = (c == 0) == (small_is_left == 1);
            ScanItem it;
            it.slot = C.slot;
            it.sub_parent = is_small ? -1 : P.slot;
            it.sub_child = is_small ? -1 : be.new_slot;
            it.valid = 1;
            it.stat.n_rows = C.count; it.stat.sum_g = C.sum_g; it.stat.sum_h = C.sum_h;
            it.out = &nodes[P.child + c].best;
            items[2 * tid + c] = it;
        }
    }
    // row groups of the histogram builds: about max_groups items in total, shared out by size
    const int total_small = block_scan_incl(small_rows, s_tmp);
    __shared__ int s_total;
    if (tid == (int)blockDim.x - 1) s_total = total_small;
    __syncthreads();
    if (tid < n_batch) {
        const int target = (int)hist_target_rows(plan, s_total, n_batch);
        groups = (small_rows + target - 1) / target;
        if (groups < 1) groups = 1;
    }
    const int gincl = block_scan_incl(groups, s_tmp);
    if (tid < n_batch) {
        const Node& S = small_is_left ? L : R;
        HistEntry e;
        e.begin = S.begin; e.count = S.count; e.buf = S.buf; e.slot = batch[tid].new_slot;
        e.item_start = gincl - groups; e.groups = groups;
        hist_entries[tid] = e;
    }
    if (tid == n_batch - 1) { hist_counts[0] = n_batch; hist_counts[1] = gincl; }
}

__global__ __launch_bounds__(256) void tree_finalize_kernel(const StepState* step, const Node* nodes,
                                                            const float* delta, int32_t* leaf_node, TreeOut out) {
    const int n = step->n_leaves;
    const double dg = (double)delta[0], dh = (double)delta[1];
    for (int l = threadIdx.x; l < out.max_leaves; l += blockDim.x) {
        if (l >= n) {
            out.t.leaf_begin[l] = 0; out.t.leaf_count[l] = 0; out.t.leaf_sum_g[l] = 0; out.t.leaf_sum_h[l] = 0;
            out.t.leaf_value_quant[l] = 0.0;
            leaf_node[l] = -1;
        }
    }
    for (int i = threadIdx.x; i < step->n_nodes; i += blockDim.x) {
        const Node S = nodes[i];
        if (S.state != 1) continue;
        const int l = S.leaf_id;
        out.t.leaf_begin[l] = S.begin; out.t.leaf_count[l] = S.count;
        out.t.leaf_sum_g[l] = S.sum_g; out.t.leaf_sum_h[l] = S.sum_h;
        out.t.leaf_value_quant[l] = (S.sum_h > 0 && dh > 0.0) ? -((double)S.sum_g * dg) / ((double)S.sum_h * dh) : 0.0;
        leaf_node[l] = i;
    }
    if (threadIdx.x == 0) {
        *out.t.n_leaves = n;
        out.t.delta[0] = delta[0]; out.t.delta[1] = delta[1];
        *out.t.hist_units = step->hist_units;
    }
}

// Copies every leaf's slice from the index buffer it ended up in to the output.
__global__ __launch_bounds__(256) void tree_gather_rows_kernel(const StepState* step, const Node* nodes,
                                                               const int32_t* __restrict__ leaf_node,
                                                               IdxSet idxs, int32_t* __restrict__ out) {
    const int l = blockIdx.y;
    if (l >= step->n_leaves) return;
    const Node S = nodes[leaf_node[l]];
    const int32_t* src = idxs.p[S.buf];
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < S.count; j += (int64_t)gridDim.x * blockDim.x)
        out[S.begin + j] = src[S.begin + j];
}

int run_grow_tree(qgbdt_ctx* ctx, const uint8_t* bins, const float* g, const float* h, const qgbdt_params* p,
                  uint32_t iteration, const qgbdt_tree* tout, int32_t* row_idx_out) {
    const int64_t N = ctx->shape.n_rows;
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    const int64_t W = (int64_t)F * nb;
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
    // Row sources: buffer 2 = the caller's matrix and the quantized gradients in original order;
    // in ordered mode buffers 0/1 are the leaf-ordered copies that the partition writes.
    RowSource rows;
    IdxSet idxs;
    const bool ordered = ctx->ordered != 0;
    for (int b = 0; b < 3; ++b) {
        rows.bins[b] = ordered ? ctx->obins[b] : bins;
        rows.gh[b] = ordered ? ctx->ogh[b] : ctx->gh;
        idxs.p[b] = ctx->idx[b];
    }
    rows.bins[BUF_ORIGINAL] = bins; rows.gh[BUF_ORIGINAL] = ctx->gh; idxs.p[BUF_ORIGINAL] = ctx->idx[0];
    const int root_buf = ordered ? BUF_ORIGINAL : 0;

    int blocks = (int)((N + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(tree_init_kernel, dim3(blocks), dim3(256), 0, ctx->stream, ctx->idx[0], N, F, ctx->step,
                       ctx->nodes, ctx->qtotals, root_buf, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                       ctx->scan_counters, ctx->hist_pool, W, plan);
    rc = launch_hist(ctx, plan, rows, idxs, false, ((uintptr_t)bins & 15) == 0,
                     ctx->hist_entries, ctx->hist_counts, ctx->hist_pool,
                     (N + plan.min_rows_per_group - 1) / plan.min_rows_per_group, ctx->step);
    if (rc != QGBDT_OK) return rc;
    rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 1, ctx->delta,
                           p->min_data_in_leaf, p->min_sum_hessian);
    if (rc != QGBDT_OK) return rc;

    const size_t plan_lds = (size_t)ctx->max_nodes * (sizeof(double) + 2 * sizeof(int)) +
                            (size_t)(14 * p->num_leaves + 24) * sizeof(int) + 64;
    const int round_cap = 4 * ctx->shape.max_leaves + 8;  // every round commits or expands at least one node
    int launched = 0;
    int to_launch = ctx->rounds_hint;
    for (;;) {
        for (int r = 0; r < to_launch; ++r) {
            hipLaunchKernelGGL(tree_plan_kernel, dim3(1), dim3(1024), plan_lds, ctx->stream, ctx->step, ctx->nodes,
                               ctx->batch, ctx->hist_counts, ctx->scan_counters, F, p->num_leaves, ctx->batch_max,
                               ctx->max_expand, out);
            rc = launch_batch_partition_count(ctx, rows);
            if (rc != QGBDT_OK) return rc;
            hipLaunchKernelGGL(tree_mid_kernel, dim3(1), dim3(1024), 0, ctx->stream, ctx->step, ctx->nodes, ctx->batch,
                               ctx->seg_counts, ctx->seg_prefix, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                               plan);
            rc = launch_batch_partition_scatter(ctx, rows);
            if (rc != QGBDT_OK) return rc;
            rc = launch_hist(ctx, plan, rows, idxs, !ordered, ordered, ctx->hist_entries,
                             ctx->hist_counts, ctx->hist_pool, plan.max_groups, ctx->step);
            if (rc != QGBDT_OK) return rc;
            rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 2 * ctx->batch_max,
                                   ctx->delta, p->min_data_in_leaf, p->min_sum_hessian);
            if (rc != QGBDT_OK) return rc;
        }
        launched += to_launch;
        // one more plan: commits what the last round made known and tells whether the tree is finished
        hipLaunchKernelGGL(tree_plan_kernel, dim3(1), dim3(1024), plan_lds, ctx->stream, ctx->step, ctx->nodes,
                           ctx->batch, ctx->hist_counts, ctx->scan_counters, F, p->num_leaves, ctx->batch_max,
                           ctx->max_expand, out);
        QG_HIP(ctx, hipGetLastError());
        QG_HIP(ctx, hipMemcpyAsync(ctx->host_state, ctx->step, sizeof(StepState), hipMemcpyDeviceToHost, ctx->stream));
        QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (ctx->host_state->done) break;
        if (launched > round_cap) return set_error(ctx, QGBDT_E_HIP, "tree growth did not finish in %d rounds", launched);
        // the trailing plan has already chosen a batch: finish that round, then continue
        rc = launch_batch_partition_count(ctx, rows);
        if (rc != QGBDT_OK) return rc;
        hipLaunchKernelGGL(tree_mid_kernel, dim3(1), dim3(1024), 0, ctx->stream, ctx->step, ctx->nodes, ctx->batch,
                           ctx->seg_counts, ctx->seg_prefix, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                           plan);
        rc = launch_batch_partition_scatter(ctx, rows);
        if (rc != QGBDT_OK) return rc;
        rc = launch_hist(ctx, plan, rows, idxs, !ordered, ordered, ctx->hist_entries,
                         ctx->hist_counts, ctx->hist_pool, plan.max_groups, ctx->step);
        if (rc != QGBDT_OK) return rc;
        rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 2 * ctx->batch_max,
                               ctx->delta, p->min_data_in_leaf, p->min_sum_hessian);
        if (rc != QGBDT_OK) return rc;
        launched += 1;
        to_launch = 3;
    }
    ctx->rounds_hint = ctx->host_state->rounds > 0 ? ctx->host_state->rounds : 1;

    hipLaunchKernelGGL(tree_finalize_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->step, ctx->nodes, ctx->delta,
                       ctx->leaf_node, out);
    int gx = (int)((N / ctx->shape.max_leaves + 255) / 256);
    if (gx < 1) gx = 1;
    if (gx > 64) gx = 64;
    hipLaunchKernelGGL(tree_gather_rows_kernel, dim3(gx, ctx->shape.max_leaves), dim3(256), 0, ctx->stream, ctx->step,
                       ctx->nodes, ctx->leaf_node, idxs, row_idx_out);
    QG_HIP(ctx, hipGetLastError());
    return launch_refit(ctx, g, h, row_idx_out, out.t.leaf_begin, out.t.leaf_count, ctx->shape.max_leaves,
                        out.t.n_leaves, out.t.leaf_value);
}

}  // namespace qgbdt
