// Stable row partition of a leaf's index slice (the set I_s of Algorithm 1) by
// bins[row][feature] <= bin.  Two passes: counts of left-going rows per segment
// (flags kept as bytes), a prefix over the segments, then an order-preserving scatter
// into another buffer.  No inter-workgroup waits: signalling between workgroups goes
// through the memory side on this chip (~1-2 us per hop), which a single-pass
// partition with look-back could not hide.  First the stand-alone form behind
// qgbdt_partition_rows (row ids only), then the batched form of grow_tree, which serves
// all nodes of a round at once and, for narrow rows, also moves the bin rows and packed
// gradients into leaf order.
#include "common.h"

namespace qgbdt {

__device__ __forceinline__ int64_t segment_len(int64_t count, int groups) {
    int64_t seg = (count + groups - 1) / groups;
    return (seg + 255) / 256 * 256;
}

__global__ void fill_i64_kernel(int64_t* p, int64_t v) {
    if (threadIdx.x == 0) *p = v;
}

__global__ void set_part_work_kernel(PartWork* w, int64_t begin, int64_t count, int feature, int bin) {
    if (threadIdx.x == 0) {
        w->begin = begin; w->count = count; w->feature = feature; w->bin = bin; w->src_buf = 0; w->zero_slot = -1;
    }
}

// Bin of (row, feature) in a row-major matrix of 8-bit (bb = 1) or 16-bit (bb = 2) bins.
__device__ __forceinline__ int bin_at(const uint8_t* __restrict__ bins, int64_t at, int bb) {
    return bb == 2 ? (int)reinterpret_cast<const uint16_t*>(bins)[at] : (int)bins[at];
}

__global__ __launch_bounds__(256) void part_count_kernel(const uint8_t* __restrict__ bins, int bb, int F,
                                                         const int32_t* __restrict__ buf0,
                                                         const int32_t* __restrict__ buf1,
                                                         const PartWork* __restrict__ work,
                                                         uint8_t* __restrict__ flags, int64_t* __restrict__ counts,
                                                         int64_t* hist_base, int64_t hist_words) {
    const PartWork wk = *work;
    if (wk.count <= 0) {
        if (threadIdx.x == 0) counts[blockIdx.x] = 0;
        return;
    }
    if (wk.zero_slot >= 0) {  // clear the histogram the smaller child will be accumulated into
        int64_t* z = hist_base + (int64_t)wk.zero_slot * hist_words;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < hist_words;
             i += (int64_t)gridDim.x * blockDim.x)
            z[i] = 0;
    }
    const int32_t* src = wk.src_buf ? buf1 : buf0;
    const int64_t seg = segment_len(wk.count, gridDim.x);
    const int64_t sbegin = (int64_t)blockIdx.x * seg;
    const int64_t send = min(wk.count, sbegin + seg);
    int cnt = 0;
    for (int64_t p = sbegin + threadIdx.x; p < send; p += blockDim.x) {
        const int64_t row = src[wk.begin + p];
        const int fl = bin_at(bins, row * F + wk.feature, bb) <= wk.bin;
        flags[wk.begin + p] = (uint8_t)fl;
        cnt += fl;
    }
    for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
    __shared__ int sc[4];
    if ((threadIdx.x & 63) == 0) sc[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) counts[blockIdx.x] = (int64_t)sc[0] + sc[1] + sc[2] + sc[3];
}

__global__ __launch_bounds__(256) void part_scatter_kernel(const int32_t* __restrict__ buf0r,
                                                           const int32_t* __restrict__ buf1r, int32_t* buf0w,
                                                           int32_t* buf1w, const PartWork* __restrict__ work,
                                                           const uint8_t* __restrict__ flags,
                                                           const int64_t* __restrict__ counts, int64_t* n_left_out) {
    const PartWork wk = *work;
    if (wk.count <= 0) return;
    const int32_t* src = wk.src_buf ? buf1r : buf0r;
    int32_t* dst = wk.src_buf ? buf0w : buf1w;
    // left rows before this segment, and in total
    int64_t before = 0, total = 0;
    for (int b = threadIdx.x; b < (int)gridDim.x; b += blockDim.x) {
        const int64_t c = counts[b];
        total += c;
        if (b < (int)blockIdx.x) before += c;
    }
    for (int o = 32; o > 0; o >>= 1) { before += __shfl_xor(before, o); total += __shfl_xor(total, o); }
    __shared__ int64_t sb[4], st[4];
    __shared__ int wl[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { sb[wave] = before; st[wave] = total; }
    __syncthreads();
    before = sb[0] + sb[1] + sb[2] + sb[3];
    total = st[0] + st[1] + st[2] + st[3];
    if (blockIdx.x == 0 && threadIdx.x == 0) *n_left_out = total;

    const int64_t seg = segment_len(wk.count, gridDim.x);
    const int64_t sbegin = (int64_t)blockIdx.x * seg;
    const int64_t send = min(wk.count, sbegin + seg);
    int64_t lpos = wk.begin + before;                      // next left slot
    int64_t rpos = wk.begin + total + (sbegin - before);   // next right slot
    for (int64_t t0 = sbegin; t0 < send; t0 += 256) {
        const int64_t p = t0 + threadIdx.x;
        const bool on = p < send;
        int fl = 0;
        int32_t v = 0;
        if (on) { fl = flags[wk.begin + p]; v = src[wk.begin + p]; }
        const unsigned long long m = __ballot(on && fl);
        const int rank = __popcll(m & ((1ull << lane) - 1ull));
        __syncthreads();
        if (lane == 0) wl[wave] = __popcll(m);
        __syncthreads();
        int lw = 0, ltile = 0;
        for (int k = 0; k < 4; ++k) { if (k < wave) lw += wl[k]; ltile += wl[k]; }
        const int pos_in_tile = wave * 64 + lane;  // order inside the tile
        if (on) {
            if (fl) dst[lpos + lw + rank] = v;
            else dst[rpos + (pos_in_tile - (lw + rank))] = v;
        }
        const int tile_n = (int)min((int64_t)256, send - t0);
        lpos += ltile;
        rpos += tile_n - ltile;
    }
}

__global__ void copy_i32_kernel(const int32_t* __restrict__ src, int32_t* __restrict__ dst, int64_t begin,
                                int64_t count) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
        dst[begin + i] = src[begin + i];
}

int launch_partition_work(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* buf0, int32_t* buf1, const PartWork* work,
                          int64_t* n_left_out, int64_t max_count) {
    const int F = ctx->shape.n_features;
    int64_t g = (max_count + 2047) / 2048;
    if (g > PART_GROUPS) g = PART_GROUPS;
    if (g < 1) g = 1;
    const int64_t W = (int64_t)F * ctx->shape.n_bins;
    hipLaunchKernelGGL(part_count_kernel, dim3((unsigned)g), dim3(256), 0, ctx->stream, bins, ctx->shape.bin_bytes, F, buf0,
                       buf1, work,
                       ctx->flags, ctx->part_counts, ctx->hist_pool, W);
    hipLaunchKernelGGL(part_scatter_kernel, dim3((unsigned)g), dim3(256), 0, ctx->stream, buf0, buf1, buf0, buf1,
                       work, ctx->flags, ctx->part_counts, n_left_out);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Stand-alone call: row_idx is reordered in place (through the context's spare buffer).
int run_partition_rows(qgbdt_ctx* ctx, const uint8_t* bins, int32_t* row_idx, int64_t begin, int64_t count,
                       int feature, int bin, int64_t* n_left_out) {
    hipLaunchKernelGGL(set_part_work_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->pwork, begin, count, feature,
                       bin);
    if (count == 0) {
        hipLaunchKernelGGL(fill_i64_kernel, dim3(1), dim3(64), 0, ctx->stream, n_left_out, (int64_t)0);
        QG_HIP(ctx, hipGetLastError());
        return QGBDT_OK;
    }
    int rc = launch_partition_work(ctx, bins, row_idx, ctx->idx[0], ctx->pwork, n_left_out, count);
    if (rc != QGBDT_OK) return rc;
    int blocks = (int)((count + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(copy_i32_kernel, dim3(blocks), dim3(256), 0, ctx->stream, ctx->idx[0], row_idx, begin, count);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}


// ---- batched partition of the nodes expanded in one round of grow_tree ---------------
//
// Work items are row segments of PART_SEG rows; segment -> (batch entry, segment of that
// node) by binary search over the entries' first-segment numbers.

// (The round's table is copied into LDS once per workgroup and searched there: through global memory the search is
// a chain of dependent loads per segment.)
__device__ __forceinline__ void load_batch(const BatchEntry* __restrict__ batch, int n_batch, BatchEntry* s_batch) {
    for (int t = threadIdx.x; t < n_batch; t += blockDim.x) s_batch[t] = batch[t];
    __syncthreads();
}
__device__ __forceinline__ int find_batch(const BatchEntry* s_batch, int n_batch, int item) {
    int lo = 0, hi = n_batch - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (s_batch[mid].seg_start <= item) lo = mid; else hi = mid - 1;
    }
    return lo;
}

// Left-going rows per segment (flags kept as bytes); on the way the histogram slots
// that this round's builds accumulate into are cleared.  In ordered mode the rows of a
// node are physically contiguous in its buffer and the bin is read at the row's position;
// otherwise it is gathered from the original matrix through the row id.
__global__ __launch_bounds__(256) void batch_part_count_kernel(RowSource rows, const uint8_t* __restrict__ bins_t, int64_t n_rows, int ordered,
                                                               int bb, int F, IdxSet idxs,
                                                               const StepState* __restrict__ step,
                                                               const BatchEntry* __restrict__ batch,
                                                               const Node* __restrict__ nodes,
                                                               uint8_t* __restrict__ flags,
                                                               int32_t* __restrict__ seg_counts, int64_t* hist_base,
                                                               int64_t hist_words) {
    if (step->done) return;
    const int n_items = step->n_part_items, n_batch = step->n_batch;
    if (n_batch <= 0) return;
    {
        int64_t* z = hist_base + (int64_t)batch[0].new_slot * hist_words;  // the new slots are consecutive
        const int64_t nz = (int64_t)n_batch * hist_words;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nz; i += (int64_t)gridDim.x * blockDim.x)
            z[i] = 0;
    }
    __shared__ int sc[4];
    __shared__ BatchEntry s_batch[TABLE_MAX];
    load_batch(batch, n_batch, s_batch);
    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const BatchEntry be = s_batch[find_batch(s_batch, n_batch, item)];
        const Node nd = nodes[be.node];
        const int32_t* src = idxs.p[nd.buf] + nd.begin;
        const uint8_t* brow = rows.bins[ordered ? nd.buf : BUF_ORIGINAL] + (ordered ? nd.begin * (int64_t)F : 0);
        // with a feature-major copy of the matrix the split feature's column is read instead: the ascending row
        // ids of a node then fall into few sectors, where the row-major matrix costs one sector per row
        const uint8_t* col = (bins_t && !ordered) ? bins_t + (int64_t)nd.best.feature * n_rows * bb : nullptr;
        const int64_t sbegin = (int64_t)(item - be.seg_start) * PART_SEG;
        const int64_t send = min(nd.count, sbegin + PART_SEG);
        const int feature = nd.best.feature, bin = nd.best.bin;
        int cnt = 0;
        for (int64_t p = sbegin + threadIdx.x; p < send; p += blockDim.x) {
            const int64_t row = (ordered || nd.buf == BUF_ORIGINAL) ? p : (int64_t)src[p];  // the root's list is the identity
            const int fl = (col ? bin_at(col, row, bb) : bin_at(brow, row * F + feature, bb)) <= bin;
            flags[nd.begin + p] = (uint8_t)fl;
            cnt += fl;
        }
        for (int o = 32; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
        __syncthreads();
        if ((threadIdx.x & 63) == 0) sc[threadIdx.x >> 6] = cnt;
        __syncthreads();
        if (threadIdx.x == 0) seg_counts[item] = sc[0] + sc[1] + sc[2] + sc[3];
    }
}

// Order-preserving scatter of every segment into the children's buffer; seg_prefix is the
// exclusive prefix of seg_counts over all segments of the round.  A workgroup takes a whole
// segment (PART_SEG = 4 x 256 rows) at once: four rows per thread are loaded together, their
// destinations follow from one round of ballots, and then (ORDERED) the bin rows move as
// dwords, eight independent loads per thread in flight, coalesced on the reading side and in
// two compacted streams on the writing side; the packed gradients move with the row ids.
template <int MODE>  // 0: row ids, 1: row ids and packed gradients, 2: those and the bin rows (ordered mode)
__global__ __launch_bounds__(256) void batch_part_scatter_kernel(RowSource rows, RowDest out, int F, IdxSet idxs,
                                                                 const StepState* __restrict__ step,
                                                                 const BatchEntry* __restrict__ batch,
                                                                 const Node* __restrict__ nodes,
                                                                 const uint8_t* __restrict__ flags,
                                                                 const int32_t* __restrict__ seg_prefix) {
    static_assert(PART_SEG == 1024, "four sub-tiles of 256 rows");
    if (step->done) return;
    const int n_items = step->n_part_items, n_batch = step->n_batch;
    __shared__ int wl[4][4];
    __shared__ int s_dpos[PART_SEG];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int dpr = F / 4;
    __shared__ BatchEntry s_batch[TABLE_MAX];
    load_batch(batch, n_batch, s_batch);
    // Segments are taken from the last to the first: the count kernel has just streamed the same
    // rows front to back, so the tail of that stream is what the memory-side cache still holds.
    for (int item = n_items - 1 - (int)blockIdx.x; item >= 0; item -= (int)gridDim.x) {
        const BatchEntry be = s_batch[find_batch(s_batch, n_batch, item)];
        const Node nd = nodes[be.node];
        const int cbuf = child_buffer(nd.buf);
        const bool identity = nd.buf == BUF_ORIGINAL;  // the root's list: row id = position, never stored
        const int32_t* src = idxs.p[nd.buf] + nd.begin;
        int32_t* dst = idxs.p[cbuf] + nd.begin;
        const int16_t* gsrc = MODE >= 1 ? rows.gh[nd.buf] + nd.begin : nullptr;
        int16_t* gdst = MODE >= 1 ? out.gh[cbuf] + nd.begin : nullptr;
        const uint8_t* bsrc = MODE == 2 ? rows.bins[nd.buf] + nd.begin * (int64_t)F : nullptr;
        uint8_t* bdst = MODE == 2 ? out.bins[cbuf] + nd.begin * (int64_t)F : nullptr;
        const int64_t sbegin = (int64_t)(item - be.seg_start) * PART_SEG;
        const int64_t send = min(nd.count, sbegin + PART_SEG);
        const int n = (int)(send - sbegin);
        const int64_t before = seg_prefix[item] - seg_prefix[be.seg_start];  // left rows in earlier segments
        const int64_t lpos0 = before;                          // first left slot of this segment (slice-relative)
        const int64_t rpos0 = nd.n_left + (sbegin - before);   // first right slot
        int fl[4], rank[4], g16[4];
        int32_t v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int r = u * 256 + threadIdx.x;
            fl[u] = 0; v[u] = 0; g16[u] = 0;
            if (r < n) {
                fl[u] = flags[nd.begin + sbegin + r];
                v[u] = identity ? (int32_t)(nd.begin + sbegin + r) : src[sbegin + r];
                if (MODE >= 1) g16[u] = gsrc[sbegin + r];
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const unsigned long long m = __ballot(fl[u] != 0);
            rank[u] = __popcll(m & ((1ull << lane) - 1ull));
            if (lane == 0) wl[u][wave] = __popcll(m);
        }
        __syncthreads();
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            int lw = 0;  // left rows of the segment in front of this wavefront's 64 rows of sub-tile u
            for (int uu = 0; uu < 4; ++uu)
                for (int w = 0; w < 4; ++w)
                    if (uu < u || (uu == u && w < wave)) lw += wl[uu][w];
            const int r = u * 256 + threadIdx.x;
            const int64_t dp = fl[u] ? lpos0 + lw + rank[u] : rpos0 + (r - (lw + rank[u]));
            if (r < n) {
                dst[dp] = v[u];
                if (MODE >= 1) gdst[dp] = (int16_t)g16[u];
                if (MODE == 2) s_dpos[r] = (int)dp;
            }
        }
        if (MODE == 2) {
            __syncthreads();
            const uint32_t* s32 = reinterpret_cast<const uint32_t*>(bsrc + sbegin * (int64_t)F);
            const int n_dw = n * dpr;
            for (int e0 = threadIdx.x; e0 < n_dw; e0 += 8 * 256) {
                uint32_t v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256;
                    v8[u] = e < n_dw ? s32[e] : 0u;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    const int e = e0 + u * 256;
                    if (e < n_dw) {
                        const int r = e / dpr, q = e - r * dpr;
                        reinterpret_cast<uint32_t*>(bdst + (int64_t)s_dpos[r] * F)[q] = v8[u];
                    }
                }
            }
        }
        __syncthreads();  // wl and s_dpos are reused by the next item
    }
}

static int batch_part_grid(const qgbdt_ctx* ctx) {
    int64_t g = ctx->max_seg;
    if (g > 2048) g = 2048;
    if (g < 1) g = 1;
    return (int)g;
}

static IdxSet idx_set(const qgbdt_ctx* ctx) {
    IdxSet s;
    s.p[0] = ctx->idx[0]; s.p[1] = ctx->idx[1]; s.p[2] = ctx->idx[2]; s.p[3] = ctx->idx[0];
    return s;
}

int launch_batch_partition_count(qgbdt_ctx* ctx, const RowSource& rows, const uint8_t* bins_t, bool ordered) {
    const int64_t W = (int64_t)ctx->shape.n_features * ctx->shape.n_bins;
    hipLaunchKernelGGL(batch_part_count_kernel, dim3(batch_part_grid(ctx)), dim3(256), 0, ctx->stream, rows, bins_t,
                       ctx->shape.n_rows, ordered ? 1 : 0, ctx->shape.bin_bytes, ctx->shape.n_features, idx_set(ctx), ctx->step, ctx->batch,
                       ctx->nodes, ctx->flags, ctx->seg_counts, ctx->hist_pool, W);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

int launch_batch_partition_scatter(qgbdt_ctx* ctx, const RowSource& rows, bool ordered) {
    RowDest out;
    for (int b = 0; b < 3; ++b) { out.bins[b] = ctx->obins[b]; out.gh[b] = ctx->ogh[b]; }
#define QG_SCATTER(MODE_)                                                                                              \
    hipLaunchKernelGGL(batch_part_scatter_kernel<MODE_>, dim3(batch_part_grid(ctx)), dim3(256), 0, ctx->stream, rows, \
                       out, ctx->shape.n_features, idx_set(ctx), ctx->step, ctx->batch, ctx->nodes, ctx->flags,       \
                       ctx->seg_prefix)
    if (ordered) QG_SCATTER(2);
    else if (rows.gh_pos) QG_SCATTER(1);
    else QG_SCATTER(0);
#undef QG_SCATTER
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Feature-major copy of a row-major bin matrix: out[f][row] = in[row][f], 32 x 32 tiles through LDS
// so that both sides are accessed along their contiguous direction.
template <typename T>
__global__ __launch_bounds__(256) void transpose_bins_kernel(const T* __restrict__ in, T* __restrict__ out, int64_t N, int F) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    const int64_t tiles_r = (N + 31) / 32;
    const int tiles_f = (F + 31) / 32;
    for (int64_t t = blockIdx.x; t < tiles_r * tiles_f; t += gridDim.x) {
        const int64_t r0 = (t / tiles_f) * 32;
        const int f0 = (int)(t % tiles_f) * 32;
        __syncthreads();
        for (int k = ty; k < 32; k += 8)
            if (r0 + k < N && f0 + tx < F) tile[k][tx] = in[(r0 + k) * F + f0 + tx];
        __syncthreads();
        for (int k = ty; k < 32; k += 8)
            if (f0 + k < F && r0 + tx < N) out[(int64_t)(f0 + k) * N + r0 + tx] = tile[tx][k];
    }
}

// The same for 8-bit bins when both the row count and the feature count are multiples of 4: 64 x 64 tiles, a
// dword (four features of a row) per load and a dword (four rows of a feature) per store.
__global__ __launch_bounds__(256) void transpose_bins4_kernel(const uint8_t* __restrict__ in, uint8_t* __restrict__ out,
                                                              int64_t N, int F) {
    __shared__ uint8_t tile[64][68];  // [row][feature]; pitch 68 keeps the dword stores of a row aligned
    const int c = threadIdx.x & 15, r = threadIdx.x >> 4;  // 16 dword columns x 16 rows per pass
    const int64_t tiles_r = (N + 63) / 64;
    const int tiles_f = (F + 63) / 64;
    for (int64_t t = blockIdx.x; t < tiles_r * tiles_f; t += gridDim.x) {
        const int64_t r0 = (t / tiles_f) * 64;
        const int f0 = (int)(t % tiles_f) * 64;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int rr = r + 16 * k;
            uint32_t v = 0u;
            if (r0 + rr < N && f0 + 4 * c < F) v = *reinterpret_cast<const uint32_t*>(in + (r0 + rr) * F + f0 + 4 * c);
            *reinterpret_cast<uint32_t*>(&tile[rr][4 * c]) = v;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int ff = r + 16 * k;  // feature of the tile; c: group of four rows
            if (f0 + ff < F && r0 + 4 * c < N) {
                const uint32_t v = (uint32_t)tile[4 * c][ff] | ((uint32_t)tile[4 * c + 1][ff] << 8) |
                                   ((uint32_t)tile[4 * c + 2][ff] << 16) | ((uint32_t)tile[4 * c + 3][ff] << 24);
                *reinterpret_cast<uint32_t*>(out + (int64_t)(f0 + ff) * N + r0 + 4 * c) = v;
            }
        }
    }
}

// Most frequent bin of every feature, from a strided sample of at most 65536 rows of the feature-major copy (the
// choice only steers which bin the histogram kernels leave out; any bin would be correct).  mfb[f] = that bin when
// it holds at least half of the sampled rows, else 0xffff.  One workgroup per feature.
template <typename T>
__global__ __launch_bounds__(256) void frequent_bins_kernel(const T* __restrict__ bins_t, int64_t N, int nb,
                                                            uint16_t* __restrict__ mfb) {
    __shared__ int cnt[1024];
    __shared__ int s_best[4], s_bin[4];
    const int f = blockIdx.x;
    for (int b = threadIdx.x; b < 1024; b += blockDim.x) cnt[b] = 0;
    __syncthreads();
    const int64_t stride = N > 65536 ? N / 65536 : 1;
    const int64_t n_s = N > 65536 ? 65536 : N;
    const T* col = bins_t + (int64_t)f * N;
    for (int64_t j = threadIdx.x; j < n_s; j += blockDim.x) {
        const int v = (int)col[j * stride];
        // lanes with equal values are counted by one of them: same-address LDS atomics serialize
        const unsigned long long active = __ballot(1);
        unsigned long long rest = active;
        const int lane = threadIdx.x & 63;
        while (rest) {
            const int lead = __ffsll((long long)rest) - 1;
            const int lv = __shfl(v, lead);
            const unsigned long long same = __ballot(v == lv) & rest;
            if (lane == lead) atomicAdd(&cnt[lv], __popcll(same));
            rest &= ~same;
        }
    }
    __syncthreads();
    int best = -1, bin = 0;
    for (int b = threadIdx.x; b < nb; b += blockDim.x)
        if (cnt[b] > best) { best = cnt[b]; bin = b; }
    for (int o = 32; o > 0; o >>= 1) {
        const int ob = __shfl_xor(best, o), obin = __shfl_xor(bin, o);
        if (ob > best || (ob == best && obin < bin)) { best = ob; bin = obin; }
    }
    if ((threadIdx.x & 63) == 0) { s_best[threadIdx.x >> 6] = best; s_bin[threadIdx.x >> 6] = bin; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k)
            if (s_best[k] > best || (s_best[k] == best && s_bin[k] < bin)) { best = s_best[k]; bin = s_bin[k]; }
        mfb[f] = (2 * (int64_t)best >= n_s) ? (uint16_t)bin : (uint16_t)0xffff;
    }
}

int launch_frequent_bins(qgbdt_ctx* ctx, const void* bins_t, uint16_t* mfb) {
    const int64_t N = ctx->shape.n_rows;
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    if (ctx->shape.bin_bytes == 2)
        hipLaunchKernelGGL(frequent_bins_kernel<uint16_t>, dim3(F), dim3(256), 0, ctx->stream,
                           static_cast<const uint16_t*>(bins_t), N, nb, mfb);
    else
        hipLaunchKernelGGL(frequent_bins_kernel<uint8_t>, dim3(F), dim3(256), 0, ctx->stream,
                           static_cast<const uint8_t*>(bins_t), N, nb, mfb);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Completes a stand-alone histogram whose kernels left out the most frequent bins: the entry of feature f's
// bin mfb[f] becomes the build's totals minus the feature's other entries.  totals: (sum g~, sum h~).
__global__ __launch_bounds__(256) void fix_frequent_bins_kernel(int64_t* hist, const int64_t* __restrict__ totals,
                                                                const uint16_t* __restrict__ mfb, int F, int nb) {
    const int f = blockIdx.x * blockDim.x + threadIdx.x;
    if (f >= F) return;
    const int mb = mfb[f];
    if (mb == 0xffff) return;
    int64_t all = 0;
    for (int b = 0; b < nb; ++b) all += hist[(int64_t)b * F + f];
    hist[(int64_t)mb * F + f] += (totals[0] * 4294967296LL + totals[1]) - all;
}

int launch_fix_frequent_bins(qgbdt_ctx* ctx, int64_t* hist, const int64_t* totals, const uint16_t* mfb) {
    const int F = ctx->shape.n_features;
    hipLaunchKernelGGL(fix_frequent_bins_kernel, dim3((F + 255) / 256), dim3(256), 0, ctx->stream, hist, totals, mfb, F,
                       ctx->shape.n_bins);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

int launch_transpose_bins(qgbdt_ctx* ctx, const void* bins, void* out) {
    const int64_t N = ctx->shape.n_rows;
    const int F = ctx->shape.n_features;
    if (ctx->shape.bin_bytes == 1 && N % 4 == 0 && F % 4 == 0 && (((uintptr_t)bins | (uintptr_t)out) & 3) == 0) {
        const int64_t tiles4 = ((N + 63) / 64) * ((F + 63) / 64);
        hipLaunchKernelGGL(transpose_bins4_kernel, dim3((unsigned)(tiles4 < 65536 ? tiles4 : 65536)), dim3(256), 0,
                           ctx->stream, static_cast<const uint8_t*>(bins), static_cast<uint8_t*>(out), N, F);
        QG_HIP(ctx, hipGetLastError());
        return QGBDT_OK;
    }
    int64_t tiles = ((N + 31) / 32) * ((F + 31) / 32);
    const int grid = (int)(tiles < 65536 ? tiles : 65536);
    if (ctx->shape.bin_bytes == 2)
        hipLaunchKernelGGL(transpose_bins_kernel<uint16_t>, dim3(grid), dim3(256), 0, ctx->stream,
                           static_cast<const uint16_t*>(bins), static_cast<uint16_t*>(out), N, F);
    else
        hipLaunchKernelGGL(transpose_bins_kernel<uint8_t>, dim3(grid), dim3(256), 0, ctx->stream,
                           static_cast<const uint8_t*>(bins), static_cast<uint8_t*>(out), N, F);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

}  // namespace qgbdt
