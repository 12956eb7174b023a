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
//   2. expands that leaf and, speculatively, other nodes with large gains -- open leaves
//      and, one level ahead, children of open leaves that are already expanded -- as
//      far as the leaf budget can still reach them: one batched partition, one batched
//      histogram build for the smaller children, one batched subtraction and split
//      search for all children.
// A speculative expansion that the replay never reaches is simply not part of the
// tree: its node stays a leaf and its row slice is untouched, because children are
// always written to another buffer (three buffers rotate with the depth, so a node's
// rows survive the expansion of its children).  Split numbers and leaf ids are
// assigned at commit time, so the result equals the sequential one bit for bit.
//
// The host enqueues whole rounds without reading anything back; after the expected
// number of rounds it reads one status word to learn whether more are needed.
#include <algorithm>

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

__global__ __launch_bounds__(256) void tree_init_kernel(int64_t N, int F, StepState* step, Node* nodes,
                                                        const int64_t* qtotals, int root_buf, HistEntry* hist_entries,
                                                        int32_t* hist_counts, ScanItem* items,
                                                        int64_t* hist0, int64_t hist_words, HistPlan plan) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    for (int64_t i = t; i < hist_words; i += stride) hist0[i] = 0;  // (the root's row list is the identity: never stored)
    if (t == 0) {
        step->done = 0; step->n_sorted = 0; step->n_nodes = 1; step->n_leaves = 1; step->n_commits = 0; step->n_expanded = 0;
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

// Exclusive prefix sum over P values in LDS (in place); every thread owns a contiguous run.
// Returns the total.
__device__ inline int block_scan_array(int* v, int P, int* tmp /*[16]*/) {
    const int per = (P + (int)blockDim.x - 1) / (int)blockDim.x;
    const int a = min((int)threadIdx.x * per, P), b = min(a + per, P);
    int local = 0;
    for (int i = a; i < b; ++i) local += v[i];
    const int incl = block_scan_incl(local, tmp);
    int run = incl - local;
    for (int i = a; i < b; ++i) { const int x = v[i]; v[i] = run; run += x; }
    __shared__ int s_scan_total;
    if (threadIdx.x == blockDim.x - 1) s_scan_total = incl;
    __syncthreads();
    return s_scan_total;
}

// Priority of an open leaf in the replay as one unsigned word: better gain rank first, then
// the lower leaf id.  Never 0.
__device__ __forceinline__ uint32_t replay_key(int rank, int leaf) {
    return ((uint32_t)(0xffff - rank) << 16) | (uint32_t)(0xffff - leaf);
}

// Commit phase and choice of the round's batch.  One workgroup of 1024 threads.
//  0. (at most 256 features) Half of the workgroup reduces the per-feature candidates of the histograms scanned
//     last to their nodes' best splits, which saves the launch that would do it.
//  1. All known nodes are kept sorted by the gain of their best split: a node's gain never changes, so
//     the order of the previous call is read back and last round's children are merged in (each
//     finds its place by a binary search and a count; old entries shift by the number of new ones
//     in front of them).  A node's rank is the number of nodes with a strictly larger gain.
//  2. One wavefront replays best-first selection: the open leaves are kept in an array indexed
//     by leaf id whose entries combine (rank, leaf id) and carry the node, so the leaf with the largest gain
//     (ties: lowest leaf id) is one wavefront-wide maximum; it is committed if it has been expanded
//     (its children become open leaves: the left one in its place, the right one as the next
//     leaf id), else the replay stops.  Only the order is recorded.
//  3. All threads write the outputs of the committed splits.
//  4. The batch is chosen by walking the sorted order (prefix sums over sorted positions).
__global__ __launch_bounds__(1024) void tree_plan_kernel(StepState* step, Node* nodes, BatchEntry* batch,
                                                         int32_t* __restrict__ sorted_idx, int32_t* hist_counts, int F,
                                                         int num_leaves, int batch_max, int max_expand, int p_max,
                                                         TreeOut out, const FeatCand* __restrict__ cand,
                                                         const ScanItem* __restrict__ scan_items) {
    // the fields of the growth state this kernel needs, in three loads that are in flight together
    const int4* sp = reinterpret_cast<const int4*>(step);
    const int4 st0 = sp[0], st1 = sp[1], st2 = sp[2];
    if (st0.x) return;  // done
    extern __shared__ unsigned char plan_lds[];
    const int n_nodes0 = st0.y;
    const int n_old = st2.z;             // nodes already in the sorted order (all but last round's children)
    const int m_new = n_nodes0 - n_old;
    const int cap = 2 * max_expand + 1;  // nodes
    const int P = n_nodes0;              // sorted positions in use
    unsigned long long* skey = reinterpret_cast<unsigned long long*>(plan_lds);  // [p_max] gain bits, sorted
    int* sidx = reinterpret_cast<int*>(skey + p_max);                            // [p_max] node at a sorted position
    unsigned long long* okeys = reinterpret_cast<unsigned long long*>(sidx + p_max);  // [p_max] the order so far
    int* oidx = reinterpret_cast<int*>(okeys + p_max);                                // [p_max]
    unsigned long long* nkey = reinterpret_cast<unsigned long long*>(oidx + p_max);   // [2*batch_max] keys of the new nodes
    // open leaves by leaf id: replay key (upper word; 0: no gain) and node (lower word)
    unsigned long long* open = nkey + 2 * batch_max;                             // [num_leaves+1]
    int* open_node = reinterpret_cast<int*>(open);                               // (the lower word of entry l is open_node[2 * l])
    int* rankof = reinterpret_cast<int*>(open + num_leaves + 1);                 // [cap] -1: cannot be split, -2: split
    int* posof = rankof + cap;                                                   // [cap] sorted position
    int* child = posof + cap;                                                    // [cap] left child, -1 if not expanded
    int* commit = child + cap;                                                   // [num_leaves] nodes committed, in order
    // per node, once the ranks are known (reuses the sorted keys): left child and the ranks of both children
    unsigned long long* ninfo = skey;                                            // [cap]; ~0: not expanded
    int* commit_lid = commit + num_leaves;                                       // [num_leaves] their leaf ids
    int* flag = reinterpret_cast<int*>(okeys);  // [P] per sorted position, reuses the old order once it is merged
    int* flag2 = flag + p_max;                  // [P]
    __shared__ int s_tmp[16];
    __shared__ int s_done, s_ncommit, s_nleaves;
    __shared__ unsigned long long s_units;
    const int tid = threadIdx.x;
    const int commits0 = st0.w, leaves0 = st0.z;
    if (tid == 0) { s_done = 0; s_ncommit = 0; s_units = 0ull; }
    // A node's sort key never changes: the gain of its best split (0 bits when it has none).  The order of
    // the nodes known at the previous call is kept in global memory; only last round's children are new.
    //
    // (matrices of at most 256 features) The new nodes' best splits are not in memory yet: the split scan has left
    // one candidate per feature, which the lower half of the workgroup reduces here instead of in a launch of its
    // own -- groups of lanes as wide as the feature count (a power of two, one wavefront at most) take a scanned
    // histogram each, write its node's best split and this kernel's entries of the node -- while the upper half
    // reads the known nodes back.  A node that has just been scanned is not expanded, and an open leaf only if it
    // is the root.
    const bool fused = cand != nullptr;
    const int half = (int)blockDim.x / 2;
    if (fused && tid < half) {
        // as few lanes per histogram as lets all histograms be reduced at once (a lane then takes several
        // features, four loads in flight): a second pass would wait for a second round of memory latencies
        const int n_scan = st2.y;  // histograms scanned in the last round
        int sub = 64;
        while (sub > 1 && (sub / 2 >= F || (half / sub) < n_scan)) sub >>= 1;
        const int per_pass = half / sub;
        const int grp = tid / sub, sl = tid % sub;
        for (int item = grp; item < n_scan; item += per_pass) {
            const ScanItem it = scan_items[item];
            double gain = 0.0;
            int feature = -1;
            if (it.valid)  // uniform over the group of lanes (a histogram that was not scanned leaves its node without a split)
                reduce_features_lanes(cand + (int64_t)item * F, F, it.stat, it.out, sl, sub, gain, feature);
            if (sl == 0) {
                const int i = (int)((reinterpret_cast<const char*>(it.out) - reinterpret_cast<const char*>(&nodes[0].best)) /
                                    (ptrdiff_t)sizeof(Node));
                const bool splittable = feature >= 0 && gain > 0.0;
                child[i] = -1;
                if (i == 0) open_node[0] = 0;
                rankof[i] = splittable ? 0 : -1;
                nkey[i - n_old] = splittable ? (unsigned long long)__double_as_longlong(gain) : 0ull;
            }
        }
    } else {
        const int first = fused ? tid - half : tid, stride = fused ? half : (int)blockDim.x;
        const int n_read = fused ? n_old : n_nodes0;
        for (int i0 = first; i0 < n_read; i0 += 2 * stride) {  // two nodes per step: their loads are in flight together
            int st[2], ex[2], ch[2], lid[2], ft[2];
            double gn[2];
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const Node* nd = &nodes[min(i0 + u * stride, n_read - 1)];
                st[u] = nd->state; ex[u] = nd->expanded; ch[u] = nd->child; lid[u] = nd->leaf_id;
                ft[u] = nd->best.feature; gn[u] = nd->best.gain;
            }
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int i = i0 + u * stride;
                if (i >= n_read) break;
                const bool splittable = ft[u] >= 0 && gn[u] > 0.0;
                const unsigned long long kb = splittable ? (unsigned long long)__double_as_longlong(gn[u]) : 0ull;
                child[i] = ex[u] ? ch[u] : -1;
                if (st[u] == 1) open_node[2 * lid[u]] = i;
                rankof[i] = st[u] == 2 ? -2 : (splittable ? 0 : -1);  // ranks are filled in below
                if (i >= n_old) nkey[i - n_old] = kb;
                else skey[i] = kb;  // by node id for now; gathered into the kept order next
            }
        }
    }
    __syncthreads();
    for (int p = tid; p < n_old; p += blockDim.x) {
        const int i = sorted_idx[p];
        oidx[p] = i;
        okeys[p] = skey[i];
    }
    __syncthreads();
    // merge: old entries keep their order and come first among equal keys; new ones follow by node id
    for (int p = tid; p < n_old; p += blockDim.x) {
        const unsigned long long kb = okeys[p];
        int c = 0;
        for (int u = 0; u < m_new; ++u) c += nkey[u] > kb ? 1 : 0;
        posof[oidx[p]] = p + c;
    }
    for (int t = (int)blockDim.x - 1 - tid; t < m_new; t += blockDim.x) {  // (from the last thread down: other wavefronts than the loop above, mostly)
        const unsigned long long kb = nkey[t];
        int lo = 0, hi = n_old;  // first old position with a smaller key
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (okeys[mid] >= kb) lo = mid + 1; else hi = mid;
        }
        int b = 0;
        for (int u = 0; u < m_new; ++u) b += (nkey[u] > kb || (nkey[u] == kb && u < t)) ? 1 : 0;
        posof[n_old + t] = lo + b;
    }
    __syncthreads();
    for (int p = tid; p < n_old; p += blockDim.x) {
        const int q = posof[oidx[p]];
        skey[q] = okeys[p]; sidx[q] = oidx[p];
    }
    __syncthreads();  // (the loop above read skey-by-id only through okeys; new entries may now overwrite it)
    for (int t = tid; t < m_new; t += blockDim.x) {
        const int q = posof[n_old + t];
        skey[q] = nkey[t]; sidx[q] = n_old + t;
    }
    __syncthreads();
    for (int p = tid; p < P; p += blockDim.x) {
        const int i = sidx[p];
        sorted_idx[p] = i;
        if (rankof[i] == 0) {
            const unsigned long long kb = skey[p];
            int r = p;
            while (r > 0 && skey[r - 1] == kb) --r;  // equal gains share a rank
            rankof[i] = r;
        }
    }
    if (tid == 0) step->n_sorted = n_nodes0;
    __syncthreads();
    for (int l = tid; l < leaves0; l += blockDim.x) {
        const int i = open_node[2 * l];
        const int r = rankof[i];
        open[l] = ((unsigned long long)(r >= 0 ? replay_key(r, l) : 0u) << 32) | (uint32_t)i;
    }
    for (int i = tid; i < n_nodes0; i += blockDim.x) {  // (overwrites the sorted keys: the ranks made from them are final)
        const int c0 = child[i];
        ninfo[i] = c0 < 0 ? ~0ull
                          : ((unsigned long long)(uint32_t)c0 << 32) | ((uint32_t)(rankof[c0] + 2) << 16) | (uint32_t)(rankof[c0 + 1] + 2);
    }
    __syncthreads();

    if (tid < 64) {
        int n_commits = commits0, n_leaves = leaves0;
        for (;;) {
            if (n_commits >= num_leaves - 1) { if (tid == 0) s_done = 1; break; }
            // a lane's best open leaf (four loads in flight per step), then the wavefront's
            uint32_t mk = 0u;
            int mn = 0;
            for (int l0 = tid; l0 < n_leaves; l0 += 256) {
                unsigned long long e[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) e[u] = (l0 + 64 * u < n_leaves) ? open[l0 + 64 * u] : 0ull;
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint32_t k = (uint32_t)(e[u] >> 32);
                    if (k > mk) { mk = k; mn = (int)(uint32_t)e[u]; }
                }
            }
            const uint32_t m = wave_max_u32(mk);
            if (m == 0u) { if (tid == 0) s_done = 1; break; }  // no open leaf has a gain > 0
            // keys are distinct (they hold the leaf id): exactly one lane has the maximum, and its node
            const int src = __builtin_amdgcn_readfirstlane(__ffsll((long long)__ballot(mk == m)) - 1);
            const int bi = __builtin_amdgcn_readlane(mn, src);
            const int wl = 0xffff - (int)(m & 0xffffu);
            const unsigned long long info = ninfo[bi];
            if (info == ~0ull) break;  // the next split is not known yet
            // commit: the left child takes the leaf's place, the right child the next leaf id
            const int c0 = (int)(info >> 32);
            const int r0 = (int)((info >> 16) & 0xffffu) - 2, r1 = (int)(info & 0xffffu) - 2;
            if (tid == 0) {
                commit[n_commits - commits0] = bi;
                commit_lid[n_commits - commits0] = wl;
                open[wl] = ((unsigned long long)(r0 >= 0 ? replay_key(r0, wl) : 0u) << 32) | (uint32_t)c0;
                open[n_leaves] = ((unsigned long long)(r1 >= 0 ? replay_key(r1, n_leaves) : 0u) << 32) | (uint32_t)(c0 + 1);
            }
            n_commits += 1; n_leaves += 1;
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
        }
        if (tid == 0) {
            s_ncommit = n_commits - commits0; s_nleaves = n_leaves;
            step->n_commits = n_commits; step->n_leaves = n_leaves;
        }
    }
    __syncthreads();
    // outputs and node states of the splits committed above
    const int n_commit = s_ncommit;
    for (int c = tid; c < n_commit; c += blockDim.x) {
        const int i = commit[c], k = commits0 + c;
        const Node nd = nodes[i];
        out.t.split_leaf[k] = commit_lid[c]; out.t.split_feature[k] = nd.best.feature; out.t.split_bin[k] = nd.best.bin;
        out.t.split_gain[k] = nd.best.gain;
        out.t.split_stats[4 * k + 0] = nd.best.left_g; out.t.split_stats[4 * k + 1] = nd.best.left_h;
        out.t.split_stats[4 * k + 2] = nd.best.right_g; out.t.split_stats[4 * k + 3] = nd.best.right_h;
        out.t.split_n_left[k] = nd.n_left;
        const int64_t nl = nd.n_left, nr = nd.count - nd.n_left;
        atomicAdd(&s_units, (unsigned long long)((nl <= nr ? nl : nr) * (int64_t)F));
        nodes[nd.child].state = 1; nodes[nd.child].leaf_id = commit_lid[c];
        nodes[nd.child + 1].state = 1; nodes[nd.child + 1].leaf_id = leaves0 + c;
    }
    __syncthreads();  // a child may itself have been committed in this call: "internal" is written last
    for (int c = tid; c < n_commit; c += blockDim.x) nodes[commit[c]].state = 2;
    if (tid == 0) step->hist_units += (int64_t)s_units;
    if (s_done) {
        if (tid == 0) {
            step->done = 1; step->n_batch = 0; step->n_part_items = 0; step->n_scan_items = 0;
            hist_counts[0] = 0; hist_counts[1] = 0;
        }
        return;
    }
    // Batch.  One expansion is certain (the leaf the replay stopped at); expansions beyond those
    // that the remaining certain ones will need may be spent on speculation.
    const int remaining = (num_leaves - 1) - (commits0 + n_commit);
    const int n_expanded0 = st1.x;
    const int spare = (max_expand - n_expanded0) - remaining;
    int want = 1 + (spare > 0 ? spare : 0);
    if (want > remaining) want = remaining;
    if (want > batch_max) want = batch_max;
    // Candidates, marked at their sorted positions: open leaves that are not expanded yet (class 0:
    // the leaf the replay stopped at is the best of them) and, one level ahead, the not yet
    // expanded children of expanded open leaves (class 1).  A node's rows outlive the expansion of
    // its children, so expanding the children of a leaf whose split is not committed yet is safe.
    // flag: 1 = committed (in this call or before), 1<<16 = class 0 candidate;  flag2: class (1 or 2), 0 none.
    for (int p = tid; p < P; p += blockDim.x) { flag[p] = 0; flag2[p] = 0; }
    __syncthreads();
    for (int c = tid; c < n_commit; c += blockDim.x) flag[posof[commit[c]]] = 1;
    for (int i = tid; i < n_nodes0; i += blockDim.x)
        if (rankof[i] == -2) flag[posof[i]] = 1;  // split in an earlier call
    const int n_leaves_now = s_nleaves;
    for (int l = tid; l < n_leaves_now; l += blockDim.x) {
        const unsigned long long e = open[l];
        if ((e >> 32) == 0ull) continue;
        const int i = (int)(uint32_t)e;
        const int c0 = child[i];
        if (c0 < 0) {
            const int p = posof[i];
            flag[p] = 1 << 16; flag2[p] = 1;
        } else {
            if (rankof[c0] >= 0 && child[c0] < 0) flag2[posof[c0]] = 2;
            if (rankof[c0 + 1] >= 0 && child[c0 + 1] < 0) flag2[posof[c0 + 1]] = 2;
        }
    }
    __syncthreads();
    // prefix over sorted positions: nodes committed in this call and class-0 candidates in front
    block_scan_array(flag, P, s_tmp);
    // A candidate is worth expanding if fewer than `remaining` nodes that can still be committed
    // have a larger gain; the best class-0 candidate always is.
    for (int p = tid; p < P; p += blockDim.x) {
        const int cls = flag2[p];
        int v = 0;
        if (cls) {
            const int before = flag[p];
            const int rank_now = p - (before & 0xffff);
            const bool pass = rank_now < remaining || (cls == 1 && (before >> 16) == 0);
            if (pass) v = (cls == 1) ? 1 : (1 << 16);
        }
        flag2[p] = v;
    }
    __syncthreads();
    for (int p = tid; p < P; p += blockDim.x) flag[p] = flag2[p];
    __syncthreads();
    const int totals = block_scan_array(flag, P, s_tmp);
    const int n0 = totals & 0xffff, n_pass = n0 + (totals >> 16);
    const int n_batch = n_pass < want ? n_pass : want;
    // order of the batch: class 0 by gain, then class 1 by gain
    for (int p = tid; p < P; p += blockDim.x) {
        const int v = flag2[p];
        if (!v) continue;
        const int o = (v & 0xffff) ? (flag[p] & 0xffff) : n0 + (flag[p] >> 16);
        if (o < n_batch) batch[o].node = sidx[p];
    }
    __syncthreads();
    __threadfence_block();
    // segments of the batched partition, new histogram slots, child ids
    int nseg = 0;
    if (tid < n_batch) nseg = (int)((nodes[batch[tid].node].count + PART_SEG - 1) / PART_SEG);
    const int incl = block_scan_incl(nseg, s_tmp);
    const int n_nodes = n_nodes0, n_slots = st1.y;
    if (tid < n_batch) {
        const int i = batch[tid].node;
        batch[tid].seg_start = incl - nseg;
        batch[tid].n_seg = nseg;
        batch[tid].new_slot = n_slots + tid;
        nodes[i].expanded = 1;
        nodes[i].child = n_nodes + 2 * tid;
    }
    if (tid == n_batch - 1) step->n_part_items = incl;
    __syncthreads();
    if (tid == 0) {
        step->n_batch = n_batch;
        step->n_nodes = n_nodes + 2 * n_batch;
        step->n_slots = n_slots + n_batch;
        step->n_expanded = n_expanded0 + n_batch;
        step->rounds = st1.w + 1;
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
    // prefix over all segments: every thread owns a contiguous run (loaded in blocks of eight
    // independent loads: one dependent load per segment would cost a memory latency each)
    const int per = (n_items + blockDim.x - 1) / blockDim.x;
    const int a = min(tid * per, n_items), b = min(a + per, n_items);
    int local = 0;
    for (int i0 = a; i0 < b; i0 += 8) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (i0 + u < b) ? seg_counts[i0 + u] : 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) local += v[u];
    }
    const int incl = block_scan_incl(local, s_tmp);
    int run = incl - local;
    for (int i0 = a; i0 < b; i0 += 8) {
        int v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (i0 + u < b) ? seg_counts[i0 + u] : 0;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            if (i0 + u < b) seg_prefix[i0 + u] = run;
            run += v[u];
        }
    }
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
    const bool identity = S.buf == BUF_ORIGINAL;  // a tree that is its root: the list was never stored
    for (int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; j < S.count; j += (int64_t)gridDim.x * blockDim.x)
        out[S.begin + j] = identity ? (int32_t)(S.begin + j) : src[S.begin + j];
}

// LDS of the plan kernel: sort keys and order of all nodes, the new nodes' keys, per-node replay state, and the
// per-leaf arrays of the replay.
static size_t plan_kernel_lds(const qgbdt_ctx* ctx, int num_leaves) {
    const int p_max = ctx->max_nodes + (ctx->max_nodes & 1);
    return (size_t)p_max * 24 + (size_t)ctx->batch_max * 16 + (size_t)ctx->max_nodes * 12 +
           (size_t)(4 * num_leaves + 8) * sizeof(int);
}

int prepare_tree_kernels(qgbdt_ctx* ctx) {
    const size_t plan_lds = plan_kernel_lds(ctx, ctx->shape.max_leaves);
    if (plan_lds + 512 > 160 * 1024)  // (the kernel's few static words come on top)
        return set_error(ctx, QGBDT_E_UNSUPPORTED, "max_leaves=%d needs %zu bytes of LDS for the growth bookkeeping (limit 160 KB)",
                         ctx->shape.max_leaves, plan_lds);
    if (plan_lds > 48 * 1024)
        QG_HIP(ctx, hipFuncSetAttribute(reinterpret_cast<const void*>(tree_plan_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)plan_lds));
    return QGBDT_OK;
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
                             ctx->delta, ctx->qtotals, ctx->ghf);
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
    // most frequent bins of the bound matrix: left out by the wide-row histogram kernels, rebuilt by the split search
    const bool skip_ok = ctx->mfb_features > 0 && ctx->bins_t && ctx->bound_bins == (const void*)bins;
    // (the large tiles that skipping makes worthwhile pay for contiguous rows only: the gathered builds of the
    // rounds keep the ordinary tiles -- 20M x 200: 212 against 197 us per launch)
    const HistPlan plan = make_hist_plan(ctx->shape, p->bits_g, p->bits_h, p->acc_width, false);
    const HistPlan root_plan = make_hist_plan_for(ctx->shape, p->bits_g, p->bits_h, p->acc_width, N, skip_ok,
                                                  ((uintptr_t)bins & 15) == 0);  // the root's build alone: contiguous rows
    const uint16_t* mfb = skip_ok ? ctx->mfb : nullptr;
    // Row sources: buffer 3 = the caller's matrix and the quantized gradients in original order;
    // buffers 0..2 are what the partition writes (see RowSource).
    RowSource rows;
    IdxSet idxs;
    // the feature-major copy serves only the matrix it was made from
    const uint8_t* bins_t = (ctx->bins_t && ctx->bound_bins == (const void*)bins) ? ctx->bins_t : nullptr;
    // Narrow rows are kept in leaf order (every level moves them) when the partition would otherwise gather a
    // sector of the row-major matrix per row; with the feature-major copy the partition is cheap without
    // moving rows, and gathering the rows of the smaller children costs less than moving all rows
    // (10.5 M x 28: 3.58 against 3.97 ms per tree).
    // Without ordered rows the packed gradients still move with the row ids (2 bytes per moved row): a gathered
    // build then reads them in sequence, which takes one of the ~2.2 cache lines per sparse narrow row away.
    // A matrix that the caches hold gathers cheaply anyway and gains nothing from the move (1 M x 28: 1.15 to
    // 1.21 against 1.16 ms per tree).
    int layout = p->row_layout;
    if (layout == QGBDT_ROWS_AUTO)
        layout = (ctx->ordered != 0 && !bins_t) ? QGBDT_ROWS_ORDERED
                 : ((int64_t)N * F * ctx->shape.bin_bytes >= (int64_t)128 << 20) ? QGBDT_ROWS_IDS_GH : QGBDT_ROWS_IDS;
    const bool ordered = layout == QGBDT_ROWS_ORDERED;
    const bool gh_lists = layout != QGBDT_ROWS_IDS;
    if (ordered && !ctx->ordered)
        return set_error(ctx, QGBDT_E_WORKSPACE, "the workspace has no room for leaf-ordered copies of the rows");
    for (int b = 0; b < 3; ++b) {
        rows.bins[b] = ordered ? ctx->obins[b] : bins;
        rows.gh[b] = gh_lists ? ctx->ogh[b] : ctx->gh;
        idxs.p[b] = ctx->idx[b];
    }
    rows.gh_pos = (gh_lists && !ordered) ? 1 : 0;
    rows.bins[BUF_ORIGINAL] = bins; rows.gh[BUF_ORIGINAL] = ctx->gh; idxs.p[BUF_ORIGINAL] = ctx->idx[0];
    // the root's rows are the original arrays under the identity list (array 0, which its great-grandchildren reuse)
    const int root_buf = BUF_ORIGINAL;

    // up to 256 features the plan kernel reduces the scan's per-feature candidates itself (one launch less per round)
    const FeatCand* fused_cand = F <= 256 ? ctx->cand : nullptr;
    int blocks = (int)((W + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(tree_init_kernel, dim3(blocks), dim3(256), 0, ctx->stream, N, F, ctx->step,
                       ctx->nodes, ctx->qtotals, root_buf, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                       ctx->hist_pool, W, root_plan);
    ctx->next_hist_is_root = 1;
    rc = launch_hist(ctx, root_plan, rows, idxs, false, ((uintptr_t)bins & 15) == 0,
                     ctx->hist_entries, ctx->hist_counts, ctx->hist_pool,
                     (N + hist_target_rows(root_plan, N, 1) - 1) / hist_target_rows(root_plan, N, 1),  // the build's row groups
                     ctx->step, mfb);
    if (rc != QGBDT_OK) return rc;
    rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 1, ctx->delta,
                           p->min_data_in_leaf, p->min_sum_hessian, ctx->cand, mfb, fused_cand == nullptr);
    if (rc != QGBDT_OK) return rc;

    const int p_max = ctx->max_nodes + (ctx->max_nodes & 1);  // even: 8-byte arrays follow 4-byte ones
    const size_t plan_lds = plan_kernel_lds(ctx, p->num_leaves);  // at most what prepare_tree_kernels allowed
    const int round_cap = 4 * ctx->shape.max_leaves + 8;  // every round commits or expands at least one node
    int launched = 0;
    int to_launch = ctx->rounds_hint;
    for (;;) {
        for (int r = 0; r < to_launch; ++r) {
            hipLaunchKernelGGL(tree_plan_kernel, dim3(1), dim3(1024), plan_lds, ctx->stream, ctx->step, ctx->nodes,
                               ctx->batch, ctx->sorted_idx, ctx->hist_counts, F, p->num_leaves, ctx->batch_max,
                               ctx->max_expand, p_max, out, fused_cand, ctx->scan_items);
            rc = launch_batch_partition_count(ctx, rows, bins_t, ordered);
            if (rc != QGBDT_OK) return rc;
            hipLaunchKernelGGL(tree_mid_kernel, dim3(1), dim3(1024), 0, ctx->stream, ctx->step, ctx->nodes, ctx->batch,
                               ctx->seg_counts, ctx->seg_prefix, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                               plan);
            rc = launch_batch_partition_scatter(ctx, rows, ordered);
            if (rc != QGBDT_OK) return rc;
            rc = launch_hist(ctx, plan, rows, idxs, !ordered, ordered, ctx->hist_entries,
                             ctx->hist_counts, ctx->hist_pool, plan.max_lanes, ctx->step, mfb);
            if (rc != QGBDT_OK) return rc;
            rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 2 * ctx->batch_max,
                                   ctx->delta, p->min_data_in_leaf, p->min_sum_hessian, ctx->cand, mfb, fused_cand == nullptr);
            if (rc != QGBDT_OK) return rc;
        }
        launched += to_launch;
        // one more plan: commits what the last round made known and tells whether the tree is finished
        hipLaunchKernelGGL(tree_plan_kernel, dim3(1), dim3(1024), plan_lds, ctx->stream, ctx->step, ctx->nodes,
                           ctx->batch, ctx->sorted_idx, ctx->hist_counts, F, p->num_leaves, ctx->batch_max,
                           ctx->max_expand, p_max, out, fused_cand, ctx->scan_items);
        QG_HIP(ctx, hipGetLastError());
        QG_HIP(ctx, hipMemcpyAsync(ctx->host_state, ctx->step, sizeof(StepState), hipMemcpyDeviceToHost, ctx->stream));
        QG_HIP(ctx, hipStreamSynchronize(ctx->stream));
        if (ctx->host_state->done) break;
        if (launched > round_cap) return set_error(ctx, QGBDT_E_HIP, "tree growth did not finish in %d rounds", launched);
        // the trailing plan has already chosen a batch: finish that round, then continue
        rc = launch_batch_partition_count(ctx, rows, bins_t, ordered);
        if (rc != QGBDT_OK) return rc;
        hipLaunchKernelGGL(tree_mid_kernel, dim3(1), dim3(1024), 0, ctx->stream, ctx->step, ctx->nodes, ctx->batch,
                           ctx->seg_counts, ctx->seg_prefix, ctx->hist_entries, ctx->hist_counts, ctx->scan_items,
                           plan);
        rc = launch_batch_partition_scatter(ctx, rows, ordered);
        if (rc != QGBDT_OK) return rc;
        rc = launch_hist(ctx, plan, rows, idxs, !ordered, ordered, ctx->hist_entries,
                         ctx->hist_counts, ctx->hist_pool, plan.max_lanes, ctx->step, mfb);
        if (rc != QGBDT_OK) return rc;
        rc = launch_scan_items(ctx, ctx->hist_pool, ctx->scan_items, &ctx->step->n_scan_items, 2 * ctx->batch_max,
                               ctx->delta, p->min_data_in_leaf, p->min_sum_hessian, ctx->cand, mfb, fused_cand == nullptr);
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
    return launch_refit(ctx, g, h, ctx->ghf, row_idx_out, out.t.leaf_begin, out.t.leaf_count, ctx->shape.max_leaves,
                        out.t.n_leaves, out.t.leaf_value);
}

}  // namespace qgbdt
