// Sibling subtraction and best-split search over integer histograms (threshold
// enumeration of Sec. 3 with the quantized gain of Sec. 4.1 eq. (gain)).
// Integer prefix sums over the packed words, fp64 gain; compiled with FMA
// contraction off so that the gain is evaluated operation by operation.
#include "split_device.h"

namespace qgbdt {

__global__ void subtract_kernel(const int64_t* __restrict__ parent, const int64_t* __restrict__ child,
                                int64_t* out, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    // a bin's child sums never exceed its parent's, so the packed words subtract field by field
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = parent[i] - child[i];
}

int launch_subtract(qgbdt_ctx* ctx, const int64_t* parent, const int64_t* child, int64_t* out, int64_t n) {
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(subtract_kernel, dim3(blocks), dim3(256), 0, ctx->stream, parent, child, out, n);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

__global__ void scan_items_from_stats_kernel(const qgbdt_leafstat* stats, int n, ScanItem* items, qgbdt_split* out,
                                             int32_t* n_items) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        ScanItem it;
        it.slot = i; it.sub_parent = -1; it.sub_child = -1; it.valid = 1; it.stat = stats[i]; it.out = out + i;
        items[i] = it;
    }
    if (i == 0) *n_items = n;
}

// One workgroup per (feature, histogram): thread b owns bin b.  Workgroup-wide
// inclusive scan of the packed words (fields cannot overflow: every prefix is
// bounded by the leaf totals), then each thread evaluates its threshold and the
// workgroup keeps the feature's best one.
__global__ __launch_bounds__(1024) void scan_kernel(int64_t* hist_base, const ScanItem* __restrict__ items,
                                                   const int32_t* __restrict__ n_items_ptr, int F, int nb,
                                                   const float* __restrict__ delta, int64_t min_data,
                                                   double min_sum_hess, FeatCand* cand_base, int glog,
                                                   const uint16_t* __restrict__ mfb) {
    const int n_items = *n_items_ptr;
    // Workgroup -> feature: histograms are [bin][feature], so the 16 features of a 128-byte line are
    // read by 16 workgroups; consecutive workgroup ids go round-robin to the 8 XCDs, so the ids are
    // dealt such that those 16 run next to each other behind one L2.
    // (Fewer per group when there are too few features to keep all XCDs busy that way.)
    const int xcd = blockIdx.x & 7, s = blockIdx.x >> 3;
    const int f = ((s >> glog) * 8 + xcd) * (1 << glog) + (s & ((1 << glog) - 1));
    if (f >= F) return;
    const int b = threadIdx.x;
    const int lane = b & 63, wave = b >> 6;
    const int64_t W = (int64_t)F * nb;
    const int64_t at = (int64_t)b * F + f;  // histograms are [bin][feature]
    const double dg = (double)delta[0], dh = (double)delta[1];
    __shared__ int64_t wtot[16];
    __shared__ double sg[16];
    __shared__ int sb[16];
    __shared__ int64_t sl[16];
    for (int item = blockIdx.y; item < n_items; item += gridDim.y) {
        const ScanItem it = items[item];
        if (!it.valid) continue;
        int64_t word = 0;
        if (b < nb) {
            if (it.sub_parent >= 0) {
                word = hist_base[it.sub_parent * W + at] - hist_base[it.sub_child * W + at];
                hist_base[it.slot * W + at] = word;
            } else {
                word = hist_base[it.slot * W + at];
            }
        }
        // inclusive scan
        int64_t pre = word;
        for (int o = 1; o < 64; o <<= 1) {
            const int64_t v = __shfl_up(pre, o);
            if (lane >= o) pre += v;
        }
        if (lane == 63) wtot[wave] = pre;
        __syncthreads();
        for (int k = 0; k < wave; ++k) pre += wtot[k];
        if (mfb != nullptr) {
            // The histogram kernels may have left out the feature's most frequent bin: the entry is then 0 and
            // what is missing from the feature's sum over all bins -- the leaf's totals are known -- belongs to
            // that bin.  (Nothing is missing when the bin was accumulated.)
            const int mb = mfb[f];
            int64_t all = 0;
            for (int k = 0; k < (int)(blockDim.x >> 6); ++k) all += wtot[k];
            const int64_t missing = (it.stat.sum_g * 4294967296LL + it.stat.sum_h) - all;
            if (mb != 0xffff && b >= mb) pre += missing;
        }

        const int64_t Gs = it.stat.sum_g, Hs = it.stat.sum_h, n = it.stat.n_rows;
        double gain = 0.0;
        int bin = -1;
        if (b + 1 < nb && Hs > 0) {
            const int64_t GL = packed_g(pre), HL = packed_h(pre);
            const int64_t GR = Gs - GL, HR = Hs - HL;
            if (HL > 0 && HR > 0) {
                const int64_t cl = count_estimate(HL, Hs, n), cr = n - cl;
                if (cl >= min_data && cr >= min_data && !((double)HL * dh < min_sum_hess) &&
                    !((double)HR * dh < min_sum_hess)) {
                    const double parent = half_loss(Gs, Hs, dg, dh);
                    const double gn = half_loss(GL, HL, dg, dh) + half_loss(GR, HR, dg, dh) - parent;
                    if (gn > 0.0) { gain = gn; bin = b; }
                }
            }
        }
        int64_t left = pre;
        // arg-max: largest gain, ties to the lowest bin
        for (int o = 32; o > 0; o >>= 1) {
            const double og = __shfl_xor(gain, o);
            const int ob = __shfl_xor(bin, o);
            const int64_t ol = __shfl_xor(left, o);
            if (ob >= 0 && (bin < 0 || og > gain || (og == gain && ob < bin))) { gain = og; bin = ob; left = ol; }
        }
        if (lane == 0) { sg[wave] = gain; sb[wave] = bin; sl[wave] = left; }
        __syncthreads();
        if (b == 0) {
            for (int k = 1; k < (int)(blockDim.x >> 6); ++k)
                if (sb[k] >= 0 && (bin < 0 || sg[k] > gain || (sg[k] == gain && sb[k] < bin))) {
                    gain = sg[k]; bin = sb[k]; left = sl[k];
                }
            FeatCand c;
            c.gain = gain; c.left = left; c.bin = bin; c.pad = 0;
            cand_base[(int64_t)item * F + f] = c;
        }
        __syncthreads();
    }
}

// The same search for histograms of at most 64 * P bins (P = 1, 2, 4) and many features.  A workgroup of 16
// wavefronts takes 16 consecutive features of an item: the [bin][16 features] tile (one 128-byte
// line per bin) is read -- and, for a subtracted sibling, written back -- with coalesced accesses
// and staged in LDS; wavefront w then scans feature w of the tile, lane l the bins l, l + 64, ...
template <int P>
__global__ __launch_bounds__(1024) void scan_tile_kernel(int64_t* hist_base, const ScanItem* __restrict__ items,
                                                         const int32_t* __restrict__ n_items_ptr, int F, int nb,
                                                         const float* __restrict__ delta, int64_t min_data,
                                                         double min_sum_hess, FeatCand* cand_base,
                                                         const uint16_t* __restrict__ mfb) {
    const int n_items = *n_items_ptr;
    const int f0 = blockIdx.x * 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t W = (int64_t)F * nb;
    const double dg = (double)delta[0], dh = (double)delta[1];
    __shared__ int64_t tile[64 * P * 17];  // [bin][feature], pitch 17 words: a wavefront's column walk spreads over the banks
    const int tf = threadIdx.x & 15, tb = threadIdx.x >> 4;  // tile loader: feature and (first) bin of this thread
    for (int item = blockIdx.y; item < n_items; item += gridDim.y) {
        const ScanItem it = items[item];
        if (!it.valid) continue;
        int64_t word[P];
#pragma unroll
        for (int j = 0; j < P; ++j) {
            const int b = tb + 64 * j;
            word[j] = 0;
            if (b < nb && f0 + tf < F) {
                const int64_t at = (int64_t)b * F + f0 + tf;
                if (it.sub_parent >= 0) word[j] = hist_base[it.sub_parent * W + at] - hist_base[it.sub_child * W + at];
                else word[j] = hist_base[it.slot * W + at];
            }
        }
        if (it.sub_parent >= 0) {
#pragma unroll
            for (int j = 0; j < P; ++j) {
                const int b = tb + 64 * j;
                if (b < nb && f0 + tf < F) hist_base[it.slot * W + (int64_t)b * F + f0 + tf] = word[j];
            }
        }
        __syncthreads();  // the previous item's tile has been read
#pragma unroll
        for (int j = 0; j < P; ++j) tile[(tb + 64 * j) * 17 + tf] = word[j];
        __syncthreads();
        const int f = f0 + wave;
        if (f >= F) continue;  // no barrier below depends on this wavefront
        int64_t pre[P];
        int64_t carry = 0;
#pragma unroll
        for (int j = 0; j < P; ++j) {
            int64_t v = tile[(lane + 64 * j) * 17 + wave];
            for (int o = 1; o < 64; o <<= 1) {
                const int64_t u = __shfl_up(v, o);
                if (lane >= o) v += u;
            }
            pre[j] = v + carry;
            carry = __shfl(pre[j], 63);
        }
        if (mfb != nullptr) {  // the feature's most frequent bin may have been left out (see scan_kernel)
            const int mb = mfb[f];
            const int64_t missing = (it.stat.sum_g * 4294967296LL + it.stat.sum_h) - carry;
#pragma unroll
            for (int j = 0; j < P; ++j)
                if (mb != 0xffff && lane + 64 * j >= mb) pre[j] += missing;
        }
        const int64_t Gs = it.stat.sum_g, Hs = it.stat.sum_h, n = it.stat.n_rows;
        double gain = 0.0;
        int bin = -1;
        int64_t left = 0;
#pragma unroll
        for (int j = 0; j < P; ++j) {  // ascending bins: strict > keeps the lowest
            const int b = lane + 64 * j;
            if (b + 1 < nb && Hs > 0) {
                const int64_t GL = packed_g(pre[j]), HL = packed_h(pre[j]);
                const int64_t GR = Gs - GL, HR = Hs - HL;
                if (HL > 0 && HR > 0) {
                    const int64_t cl = count_estimate(HL, Hs, n), cr = n - cl;
                    if (cl >= min_data && cr >= min_data && !((double)HL * dh < min_sum_hess) &&
                        !((double)HR * dh < min_sum_hess)) {
                        const double parent = half_loss(Gs, Hs, dg, dh);
                        const double gn = half_loss(GL, HL, dg, dh) + half_loss(GR, HR, dg, dh) - parent;
                        if (gn > 0.0 && gn > gain) { gain = gn; bin = b; left = pre[j]; }
                    }
                }
            }
        }
        for (int o = 32; o > 0; o >>= 1) {  // arg-max: largest gain, ties to the lowest bin
            const double og = __shfl_xor(gain, o);
            const int ob = __shfl_xor(bin, o);
            const int64_t ol = __shfl_xor(left, o);
            if (ob >= 0 && (bin < 0 || og > gain || (og == gain && ob < bin))) { gain = og; bin = ob; left = ol; }
        }
        if (lane == 0) {
            FeatCand c;
            c.gain = gain; c.left = left; c.bin = bin; c.pad = 0;
            cand_base[(int64_t)item * F + f] = c;
        }
    }
}

// Per-feature candidates -> best split of every scanned histogram, one wavefront per histogram.
__global__ __launch_bounds__(256) void reduce_items_kernel(const FeatCand* __restrict__ cand_base,
                                                           const ScanItem* __restrict__ items,
                                                           const int32_t* __restrict__ n_items_ptr, int F) {
    const int n_items = *n_items_ptr;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (F > 256) {
        // many features: the four wavefronts share an item (a quarter of the features each, ascending)
        __shared__ FeatCand part[4];
        __shared__ int pf[4];
        for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
            const ScanItem it = items[item];
            if (!it.valid) continue;  // uniform over the workgroup
            const FeatCand* cand = cand_base + (int64_t)item * F;
            const int q = (F + 3) / 4, fb = wave * q, fe = min(F, fb + q);
            double bg = 0.0;
            int bf = -1;
            for (int f = fb + lane; f < fe; f += 64) {
                const FeatCand c = cand[f];
                if (c.bin >= 0 && (c.gain > bg)) { bg = c.gain; bf = f; }
            }
            for (int o = 32; o > 0; o >>= 1) {
                const double og = __shfl_xor(bg, o);
                const int of = __shfl_xor(bf, o);
                if (of >= 0 && (bf < 0 || og > bg || (og == bg && of < bf))) { bg = og; bf = of; }
            }
            __syncthreads();
            if (lane == 0) {
                pf[wave] = bf;
                if (bf >= 0) part[wave] = cand[bf];
            }
            __syncthreads();
            if (threadIdx.x == 0) {
                int best = -1;
                for (int k = 0; k < 4; ++k)  // ascending feature ranges: strict > keeps the lowest feature
                    if (pf[k] >= 0 && (best < 0 || part[k].gain > part[best].gain)) best = k;
                qgbdt_split sp;
                sp.gain = 0.0; sp.feature = -1; sp.bin = -1;
                sp.left_g = sp.left_h = sp.right_g = sp.right_h = sp.left_count = 0;
                if (best >= 0) {
                    const FeatCand c = part[best];
                    sp.gain = c.gain; sp.feature = pf[best]; sp.bin = c.bin;
                    sp.left_g = packed_g(c.left); sp.left_h = packed_h(c.left);
                    sp.right_g = it.stat.sum_g - sp.left_g; sp.right_h = it.stat.sum_h - sp.left_h;
                    sp.left_count = count_estimate(sp.left_h, it.stat.sum_h, it.stat.n_rows);
                }
                *it.out = sp;
            }
        }
        return;
    }
    for (int item = blockIdx.x * 4 + wave; item < n_items; item += gridDim.x * 4) {
        const ScanItem it = items[item];
        if (!it.valid) continue;
        reduce_features_wave(cand_base + (int64_t)item * F, F, it.stat, it.out, lane);
    }
}

int launch_scan_items(qgbdt_ctx* ctx, int64_t* hist_base, const ScanItem* items, const int32_t* n_items, int max_items,
                      const float* delta, int min_data, double min_sum_hess, FeatCand* cand, const uint16_t* mfb,
                      bool reduce) {
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    int threads = 64;
    while (threads < nb) threads <<= 1;
    // a workgroup walks the items gy apart one after the other, each a chain of dependent loads:
    // enough workgroups that few items queue behind each other (about 32 K wavefronts at most)
    int gy = 32768 / (F * (threads / 64));
    if (gy < 2) gy = 2;
    if (gy > max_items) gy = max_items;
    if (gy < 1) gy = 1;
    int glog = 0;  // features per XCD group: 16 (one 128-byte line) when F >= 128, fewer for narrow matrices
    while (glog < 4 && (16 << glog) <= F) ++glog;
    if (nb <= 256 && F >= 64) {
        const int gx = (F + 15) / 16;
        gy = 2048 / gx;
        if (gy < 2) gy = 2;
        if (gy > max_items) gy = max_items;
        if (gy < 1) gy = 1;
#define QG_SCAN_TILE(P_)                                                                                          \
    hipLaunchKernelGGL(scan_tile_kernel<P_>, dim3(gx, gy), dim3(1024), 0, ctx->stream, hist_base, items, n_items, \
                       F, nb, delta, (int64_t)min_data, min_sum_hess, cand, mfb)
        if (nb <= 64) QG_SCAN_TILE(1);
        else if (nb <= 128) QG_SCAN_TILE(2);
        else QG_SCAN_TILE(4);
#undef QG_SCAN_TILE
    } else {
        const int per = 8 << glog;
        const int gx = (F + per - 1) / per * per;
        hipLaunchKernelGGL(scan_kernel, dim3(gx, gy), dim3(threads), 0, ctx->stream, hist_base, items, n_items, F, nb,
                           delta, (int64_t)min_data, min_sum_hess, cand, glog, mfb);
    }
    if (reduce) {  // (tree growth leaves the candidates of narrow matrices to its next kernel)
        int gr = F > 256 ? max_items : (max_items + 3) / 4;
        if (gr > 64) gr = 64;
        hipLaunchKernelGGL(reduce_items_kernel, dim3(gr), dim3(256), 0, ctx->stream, cand, items, n_items, F);
    }
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Stand-alone search over n_hists contiguous histograms, in batches of the item table it is given.
int run_find_best_splits(qgbdt_ctx* ctx, const int64_t* hist, int n_hists, const qgbdt_leafstat* stats,
                         const float* delta, int min_data, double min_sum_hess, qgbdt_split* out, int cap,
                         ScanItem* items, FeatCand* cand, int32_t* n_items) {
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    const int64_t W = (int64_t)F * nb;
    for (int h0 = 0; h0 < n_hists; h0 += cap) {
        const int n = (n_hists - h0 < cap) ? (n_hists - h0) : cap;
        hipLaunchKernelGGL(scan_items_from_stats_kernel, dim3((n + 63) / 64), dim3(64), 0, ctx->stream, stats + h0, n,
                           items, out + h0, n_items);
        int rc = launch_scan_items(ctx, const_cast<int64_t*>(hist) + h0 * W, items, n_items, n, delta,
                                   min_data, min_sum_hess, cand);
        if (rc != QGBDT_OK) return rc;
    }
    return QGBDT_OK;
}

}  // namespace qgbdt
