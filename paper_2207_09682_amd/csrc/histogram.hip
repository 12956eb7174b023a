// Histogram construction (Algorithm 1 with quantized gradients, Sec. 4.1) with
// workgroup-local packed accumulators in LDS merged into the leaf's total
// histogram by 64-bit integer atomics (hierarchical buffers of Sec. 6.1, packed
// gradient|hessian words of Sec. 6.2, width rule of Sec. 7.4.3).
//
// Bound by HBM: per row one F-byte bin row, one 2-byte packed (g~,h~) and, for a
// non-root leaf, one 4-byte row id are read once; the only other traffic is the
// merge of F*n_bins packed words per workgroup chunk.
//
// Mapping.  The bin matrix is row-major.  A wavefront covers `rows_per_it`
// consecutive rows per iteration: lane -> (row r, dword q of the row's feature
// tile), so a wavefront reads rows_per_it * ft contiguous (or row-gathered) bytes
// with one dword load per lane, and the lane's (r, q) never change.  Each dword
// holds four features; the four LDS atomics of a lane are issued in an order
// rotated by (r + q/8), and the local histogram is laid out [bin][feature] with a
// row pitch that is a multiple of 32 words for narrow tiles, so that in one
// atomic instruction lanes of different features fall into different LDS banks.
#include "common.h"

namespace qgbdt {

__global__ void fill_zero_kernel(int64_t* p, int64_t n) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) p[i] = 0;
}

int launch_fill_zero(qgbdt_ctx* ctx, int64_t* p, int64_t n_words) {
    int blocks = (int)((n_words + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(blocks), dim3(256), 0, ctx->stream, p, n_words);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

// Expands the per-row int16 (g~ high byte, h~ low byte) into the packed word that
// is added to a bin: g~ * 2^W + h~.
template <int W>
struct Acc;
template <>
struct Acc<16> {
    using word = uint32_t;
    static __device__ __forceinline__ word expand(int ghv) { return (word)((ghv >> 8) * 65536 + (ghv & 0xff)); }
    static __device__ __forceinline__ void add(word* p, word v) { atomicAdd(p, v); }
    static __device__ __forceinline__ int64_t widen(word v) {
        const int64_t G = (int32_t)v >> 16;
        const int64_t H = v & 0xffffu;
        return G * 4294967296LL + H;
    }
};
template <>
struct Acc<32> {
    using word = unsigned long long;
    static __device__ __forceinline__ word expand(int ghv) {
        return (word)((int64_t)(ghv >> 8) * 4294967296LL + (int64_t)(ghv & 0xff));
    }
    static __device__ __forceinline__ void add(word* p, word v) { atomicAdd(p, v); }
    static __device__ __forceinline__ int64_t widen(word v) { return (int64_t)v; }
};

template <int W>
__global__ __launch_bounds__(256) void hist_kernel(const uint8_t* __restrict__ bins, const int16_t* __restrict__ gh,
                                                   const int32_t* __restrict__ idx0,
                                                   const int32_t* __restrict__ idx1,
                                                   const HistWork* __restrict__ work, int64_t* hist_base, int F,
                                                   int nb, HistPlan plan, StepState* step) {
    using word = typename Acc<W>::word;
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);

    const HistWork wk = *work;
    if (wk.count <= 0) return;
    if (step && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        step->hist_units += wk.count * (int64_t)F;
        if (wk.use_idx) step->prof_rows_idx += wk.count; else step->prof_rows_contig += wk.count;
        step->prof_launches += 1;
    }
    int64_t rows_per_group = (wk.count + gridDim.x - 1) / gridDim.x;
    if (rows_per_group < plan.min_rows_per_group) rows_per_group = plan.min_rows_per_group;
    const int64_t gbegin = (int64_t)blockIdx.x * rows_per_group;
    if (gbegin >= wk.count) return;
    const int64_t gend = min(wk.count, gbegin + rows_per_group);

    const int f0 = blockIdx.y * plan.ft;
    const int ft = min(plan.ft, F - f0);
    const int ftp = plan.ftp;
    const int lds_words = nb * ftp;
    int64_t* hist = hist_base + (int64_t)wk.slot * F * nb;
    const int32_t* idx = wk.use_idx ? (wk.buf ? idx1 : idx0) : nullptr;

    for (int w = threadIdx.x; w < lds_words; w += blockDim.x) lds[w] = 0;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, n_waves = blockDim.x >> 6;
    const int q = lane % plan.dpr, r = lane / plan.dpr;
    const bool lane_on = (r < plan.rows_per_it) && (4 * q < ft);
    const int rot = (q >> 3) + r;
    int sh[4], fl[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int c = (k + rot) & 3;
        sh[k] = 8 * c;
        fl[k] = 4 * q + c;
    }
    const int64_t row_stride = (int64_t)n_waves * plan.rows_per_it;
    const uint8_t* col = bins + f0 + 4 * q;

    for (int64_t cbegin = gbegin; cbegin < gend; cbegin += plan.chunk_rows) {
        const int64_t cend = min(gend, cbegin + (int64_t)plan.chunk_rows);
        __syncthreads();
        if (lane_on) {
            for (int64_t p0 = cbegin + (int64_t)wave * plan.rows_per_it + r; p0 < cend; p0 += 4 * row_stride) {
                uint32_t d[4];
                int gv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t p = p0 + u * row_stride;
                    d[u] = 0; gv[u] = 0;
                    if (p < cend) {
                        const int64_t i = idx ? (int64_t)idx[wk.begin + p] : wk.begin + p;
                        d[u] = *reinterpret_cast<const uint32_t*>(col + i * F);
                        gv[u] = gh[i];
                    }
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    if (p0 + u * row_stride < cend) {
                        const word v = Acc<W>::expand(gv[u]);
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            const uint32_t b = (d[u] >> sh[k]) & 0xffu;
                            Acc<W>::add(&lds[b * ftp + fl[k]], v);
                        }
                    }
                }
            }
        }
        __syncthreads();
        // merge the local bins into the total histogram and clear them
        const int n_words = ft * nb;
        for (int w = threadIdx.x; w < n_words; w += blockDim.x) {
            const int f = w / nb, b = w - f * nb;
            const word v = lds[b * ftp + f];
            if (v != 0) {
                lds[b * ftp + f] = 0;
                atomicAdd(reinterpret_cast<unsigned long long*>(hist + (int64_t)(f0 + f) * nb + b),
                          (unsigned long long)Acc<W>::widen(v));
            }
        }
    }
}

// Any feature count (no alignment assumption): one byte load per (row, feature).
template <int W>
__global__ __launch_bounds__(256) void hist_generic_kernel(const uint8_t* __restrict__ bins,
                                                           const int16_t* __restrict__ gh,
                                                           const int32_t* __restrict__ idx0,
                                                           const int32_t* __restrict__ idx1,
                                                           const HistWork* __restrict__ work, int64_t* hist_base,
                                                           int F, int nb, HistPlan plan, StepState* step) {
    using word = typename Acc<W>::word;
    extern __shared__ unsigned char lds_raw[];
    word* lds = reinterpret_cast<word*>(lds_raw);
    const HistWork wk = *work;
    if (wk.count <= 0) return;
    if (step && blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) {
        step->hist_units += wk.count * (int64_t)F;
        if (wk.use_idx) step->prof_rows_idx += wk.count; else step->prof_rows_contig += wk.count;
        step->prof_launches += 1;
    }
    int64_t rows_per_group = (wk.count + gridDim.x - 1) / gridDim.x;
    if (rows_per_group < plan.min_rows_per_group) rows_per_group = plan.min_rows_per_group;
    const int64_t gbegin = (int64_t)blockIdx.x * rows_per_group;
    if (gbegin >= wk.count) return;
    const int64_t gend = min(wk.count, gbegin + rows_per_group);
    const int f0 = blockIdx.y * plan.ft;
    const int ft = min(plan.ft, F - f0);
    const int n_words = ft * nb;
    int64_t* hist = hist_base + (int64_t)wk.slot * F * nb;
    const int32_t* idx = wk.use_idx ? (wk.buf ? idx1 : idx0) : nullptr;
    for (int w = threadIdx.x; w < n_words; w += blockDim.x) lds[w] = 0;
    for (int64_t cbegin = gbegin; cbegin < gend; cbegin += plan.chunk_rows) {
        const int64_t cend = min(gend, cbegin + (int64_t)plan.chunk_rows);
        __syncthreads();
        const int64_t n_el = (cend - cbegin) * ft;
        for (int64_t e = threadIdx.x; e < n_el; e += blockDim.x) {
            const int64_t p = cbegin + e / ft;
            const int f = (int)(e % ft);
            const int64_t i = idx ? (int64_t)idx[wk.begin + p] : wk.begin + p;
            const uint32_t b = bins[i * F + f0 + f];
            Acc<W>::add(&lds[f * nb + b], Acc<W>::expand(gh[i]));
        }
        __syncthreads();
        for (int w = threadIdx.x; w < n_words; w += blockDim.x) {
            const word v = lds[w];
            if (v != 0) {
                lds[w] = 0;
                atomicAdd(reinterpret_cast<unsigned long long*>(hist + (int64_t)f0 * nb + w),
                          (unsigned long long)Acc<W>::widen(v));
            }
        }
    }
}

static int64_t rows_fitting(int bits_g, int bits_h, int w) {
    const int64_t kg = (1 << (bits_g - 1)) - 1, kh = (1 << bits_h) - 2;
    const int64_t a = (((int64_t)1 << (w - 1)) - 1) / kg;
    const int64_t b = (((int64_t)1 << w) - 1) / kh;
    return a < b ? a : b;
}

int64_t max_rows_for_width(int bits_g, int bits_h, int w) { return rows_fitting(bits_g, bits_h, w); }

// Chooses tile width, accumulator width and launch shape for a problem shape.
HistPlan make_hist_plan(const qgbdt_shape& s, int bits_g, int bits_h, int acc_width) {
    HistPlan p{};
    const int F = s.n_features, nb = s.n_bins;
    const int64_t n16 = rows_fitting(bits_g, bits_h, 16);
    int w = acc_width;
    if (w == 0) w = (n16 >= 1024) ? 16 : 32;  // a 16|16 chunk must amortise its merge
    const int wbytes = (w == 16) ? 4 : 8;
    const int lds_budget = 64 * 1024;
    p.threads = 256;
    const bool fast = (F % 4 == 0);
    if (fast) {
        // candidates in order of preference: the whole row when it is narrow, then wide tiles
        // (whole cache lines per row), small tiles only when nothing else fits the LDS budget
        const int cands[] = {(F <= 64) ? F : 0, 128, 96, 64, 48, 40, 32, 24, 16, 8, 4};
        int best_ft = 0;
        for (int pass = 0; pass < 2 && best_ft == 0; ++pass) {
            double best_score = -1.0;
            for (int c = 0; c < 11; ++c) {
                const int ft = cands[c];
                if (ft <= 0 || ft > F || ft % 4) continue;
                if (pass == 0 && ft < 32 && ft != F) continue;
                const int ftp = (ft <= 32) ? 32 : ft;
                if ((int64_t)ftp * nb * wbytes > lds_budget) continue;
                const int dpr = ft / 4;
                const int rpi = 64 / dpr;
                const int tiles = (F + ft - 1) / ft;
                const double score = ((double)(rpi * dpr) / 64.0) * ((double)F / ((double)tiles * ft));
                if (score > best_score + 1e-9) { best_score = score; best_ft = ft; }
            }
        }
        if (best_ft == 0) best_ft = 4;
        p.ft = best_ft;
        p.ftp = (best_ft <= 32) ? 32 : best_ft;
        p.dpr = best_ft / 4;
        p.rows_per_it = 64 / p.dpr;
        p.lds_bytes = p.ftp * nb * wbytes;
    } else {
        int ft = lds_budget / (nb * wbytes);
        if (ft > F) ft = F;
        if (ft < 1) ft = 1;
        p.ft = ft; p.ftp = ft; p.dpr = 0; p.rows_per_it = 0;
        p.lds_bytes = ft * nb * wbytes;
    }
    p.n_tiles = (F + p.ft - 1) / p.ft;
    const int64_t lim = (w == 16) ? n16 : rows_fitting(bits_g, bits_h, 32);
    p.chunk_rows = (int32_t)((lim > 0x40000000LL) ? 0x40000000LL : lim);
    if (p.chunk_rows < 1) p.chunk_rows = 1;
    p.min_rows_per_group = 2048;
    int per_cu = (160 * 1024) / (p.lds_bytes > 0 ? p.lds_bytes : 1);
    if (per_cu > 8) per_cu = 8;
    if (per_cu < 1) per_cu = 1;
    int groups = (256 * per_cu) / p.n_tiles;
    if (groups < 1) groups = 1;
    p.max_groups = groups;
    p.acc_width = w;
    return p;
}

int launch_hist(qgbdt_ctx* ctx, const HistPlan& plan, const uint8_t* bins, const int16_t* gh,
                const int32_t* idx0, const int32_t* idx1, const HistWork* work, int64_t* hist_base,
                int64_t max_count, StepState* step) {
    const int F = ctx->shape.n_features, nb = ctx->shape.n_bins;
    int64_t groups = (max_count + plan.min_rows_per_group - 1) / plan.min_rows_per_group;
    if (groups > plan.max_groups) groups = plan.max_groups;
    if (groups < 1) groups = 1;
    dim3 grid((unsigned)groups, (unsigned)plan.n_tiles), block(plan.threads);
    const bool fast = (F % 4 == 0);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ctx->profiling && ctx->ev_used + 2 <= ctx->ev_cap) {
        e0 = ctx->ev[ctx->ev_used++]; e1 = ctx->ev[ctx->ev_used++];
        QG_HIP(ctx, hipEventRecord(e0, ctx->stream));
    }
    if (plan.acc_width == 16) {
        if (fast)
            hipLaunchKernelGGL(hist_kernel<16>, grid, block, plan.lds_bytes, ctx->stream, bins, gh, idx0, idx1, work,
                               hist_base, F, nb, plan, step);
        else
            hipLaunchKernelGGL(hist_generic_kernel<16>, grid, block, plan.lds_bytes, ctx->stream, bins, gh, idx0,
                               idx1, work, hist_base, F, nb, plan, step);
    } else {
        if (fast)
            hipLaunchKernelGGL(hist_kernel<32>, grid, block, plan.lds_bytes, ctx->stream, bins, gh, idx0, idx1, work,
                               hist_base, F, nb, plan, step);
        else
            hipLaunchKernelGGL(hist_generic_kernel<32>, grid, block, plan.lds_bytes, ctx->stream, bins, gh, idx0,
                               idx1, work, hist_base, F, nb, plan, step);
    }
    QG_HIP(ctx, hipGetLastError());
    if (e1) {
        QG_HIP(ctx, hipEventRecord(e1, ctx->stream));
        ctx->prof_launches += 1;
    }
    return QGBDT_OK;
}

}  // namespace qgbdt
