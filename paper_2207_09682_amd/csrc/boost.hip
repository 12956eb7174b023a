// The two steps around a tree that close the boosting loop on the device (Sec. 3): the loss
// derivatives g_i, h_i of the current predictions (binary cross-entropy) and the prediction
// update with the new tree's leaf values.  Both are HBM-bound streaming / gather kernels.
#include "common.h"

namespace qgbdt {

// p = 1 / (1 + exp(-s)) in fp64 from the fp32 score, g = p - y, h = p (1 - p), each rounded
// once to fp32: 16 bytes of traffic per row hide the fp64 arithmetic.
__device__ __forceinline__ void logistic_one(float s, float y, float& g, float& h) {
    const double p = 1.0 / (1.0 + exp(-(double)s));
    g = (float)(p - (double)y);
    h = (float)(p * (1.0 - p));
}

template <bool VEC>
__global__ __launch_bounds__(256) void logistic_grad_kernel(const float* __restrict__ score,
                                                            const float* __restrict__ label, int64_t n,
                                                            float* __restrict__ g, float* __restrict__ h) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (VEC) {  // all four arrays 16-byte aligned
        const int64_t n4 = n >> 2;
        for (int64_t i = t0; i < n4; i += stride) {
            const float4 s = reinterpret_cast<const float4*>(score)[i], y = reinterpret_cast<const float4*>(label)[i];
            float4 go, ho;
            logistic_one(s.x, y.x, go.x, ho.x); logistic_one(s.y, y.y, go.y, ho.y);
            logistic_one(s.z, y.z, go.z, ho.z); logistic_one(s.w, y.w, go.w, ho.w);
            reinterpret_cast<float4*>(g)[i] = go;
            reinterpret_cast<float4*>(h)[i] = ho;
        }
        const int64_t r = (n4 << 2) + t0;
        if (r < n) logistic_one(score[r], label[r], g[r], h[r]);
    } else {
        for (int64_t i = t0; i < n; i += stride) logistic_one(score[i], label[i], g[i], h[i]);
    }
}

// score[row] += (float)(lr * value[leaf]) for the rows of every leaf: block (part, leaf) takes
// a contiguous part of the leaf's slice of the leaf-ordered row list.
__global__ __launch_bounds__(256) void update_scores_kernel(float* __restrict__ score,
                                                            const int32_t* __restrict__ row_idx,
                                                            const int64_t* __restrict__ leaf_begin,
                                                            const int64_t* __restrict__ leaf_count,
                                                            const double* __restrict__ leaf_value,
                                                            const int32_t* __restrict__ n_leaves_dev, double lr) {
    const int l = blockIdx.y;
    if (n_leaves_dev && l >= *n_leaves_dev) return;
    const int64_t begin = leaf_begin[l], count = leaf_count[l];
    const float d = (float)(lr * leaf_value[l]);
    const int64_t a = count * blockIdx.x / gridDim.x, b = count * (blockIdx.x + 1) / gridDim.x;
    for (int64_t j = a + threadIdx.x; j < b; j += blockDim.x) {
        const int64_t i = row_idx[begin + j];
        score[i] += d;  // every row belongs to exactly one leaf: no two threads touch the same element
    }
}

// Pairwise ranking loss with NDCG weights (lambdarank): one workgroup per query of `group`
// consecutive rows.  Ranks (by score, ties by position), discounts, gains and the ideal DCG are
// formed in LDS; then every thread owns documents and walks all partners, so its sums need no
// atomics and have a fixed order.  For a pair (a, b) with rel_a > rel_b:
//   rho = 1 / (1 + exp(s_a - s_b)),  w = |gain_a - gain_b| |disc_a - disc_b| / maxDCG,
//   g_a -= rho w, g_b += rho w, h_a += rho (1 - rho) w, h_b += rho (1 - rho) w;  fp64, rounded once.
// The path is bound by fp64 arithmetic (group^2 pair terms per query), so the per-pair work is
// kept small: exp(s_a - s_b) = exp(s_a - c) exp(c - s_b) with c the middle of the query's score
// range (two exp per document instead of one per pair; queries whose range would overflow that
// take the direct form), the reciprocal by the hardware estimate and two Newton steps, the
// division by maxDCG once per document, and pairs of equal relevance drop out through w = 0.
__device__ __forceinline__ double recip_newton(double d) {
    double y = __builtin_amdgcn_rcp(d);
    y = fma(fma(-d, y, 1.0), y, y);
    y = fma(fma(-d, y, 1.0), y, y);
    return y;
}

__global__ __launch_bounds__(128) void lambdarank_grad_kernel(const float* __restrict__ score,
                                                              const float* __restrict__ label, int64_t n, int group,
                                                              float* __restrict__ g, float* __restrict__ h) {
    extern __shared__ __align__(16) double lr_lds[];
    double* s = lr_lds;                                        // [group] scores
    double* r = s + group;                                     // [group] relevance grades
    double2* ee = reinterpret_cast<double2*>(r + group);       // [group] exp(s - c), exp(c - s)
    double2* gd = ee + group;                                  // [group] gain, discount
    __shared__ double wsum[2], wmax[2], wmin[2];
    const int tid = threadIdx.x;
    const int64_t n_queries = (n + group - 1) / group;
    for (int64_t q = blockIdx.x; q < n_queries; q += gridDim.x) {
        const int64_t q0 = q * group;
        const int m = (int)min((int64_t)group, n - q0);
        __syncthreads();  // the previous query's values are no longer read
        double smax = -1.0e308, smin = 1.0e308;
        for (int k = tid; k < m; k += blockDim.x) {
            const double sk = (double)score[q0 + k];
            s[k] = sk;
            r[k] = (double)label[q0 + k];
            smax = fmax(smax, sk); smin = fmin(smin, sk);
        }
        for (int o = 32; o > 0; o >>= 1) { smax = fmax(smax, __shfl_xor(smax, o)); smin = fmin(smin, __shfl_xor(smin, o)); }
        if ((tid & 63) == 0) { wmax[tid >> 6] = smax; wmin[tid >> 6] = smin; }
        __syncthreads();
        smax = fmax(wmax[0], wmax[1]); smin = fmin(wmin[0], wmin[1]);
        const double c = 0.5 * (smax + smin);
        const bool direct = !((smax - smin) < 690.0);  // the product of two factors reaches exp(range): must stay finite (also catches NaN scores)
        double part = 0.0;
        for (int k = tid; k < m; k += blockDim.x) {
            int rank = 0, irank = 0;
            const double sk = s[k], rk = r[k];
            for (int j = 0; j < m; ++j) {
                rank += (s[j] > sk || (s[j] == sk && j < k)) ? 1 : 0;
                irank += (r[j] > rk || (r[j] == rk && j < k)) ? 1 : 0;
            }
            const double gk = exp2(rk) - 1.0;
            gd[k] = make_double2(gk, 1.0 / log2((double)rank + 2.0));
            if (!direct) ee[k] = make_double2(exp(sk - c), exp(c - sk));
            part += gk / log2((double)irank + 2.0);
        }
        for (int o = 32; o > 0; o >>= 1) part += __shfl_xor(part, o);
        if ((tid & 63) == 0) wsum[tid >> 6] = part;
        __syncthreads();
        const double max_dcg = wsum[0] + wsum[1];
        for (int k = tid; k < m; k += blockDim.x) {
            double G = 0.0, H = 0.0;
            if (max_dcg > 0.0) {
                const double2 gdk = gd[k];
                if (!direct) {
                    const double2 ek = ee[k];
                    for (int j = 0; j < m; ++j) {
                        const double2 gdj = gd[j], ej = ee[j];
                        const bool up = gdk.x > gdj.x;  // k is the more relevant one of the pair
                        const double w = fabs(gdk.x - gdj.x) * fabs(gdk.y - gdj.y);  // 0 for equal relevance
                        const double x = up ? ek.x * ej.y : ej.x * ek.y;          // exp(s_hi - s_lo)
                        const double rho = recip_newton(1.0 + x);
                        const double rw = rho * w;
                        G += up ? -rw : rw;
                        H = fma(1.0 - rho, rw, H);
                    }
                } else {
                    const double sk = s[k];
                    for (int j = 0; j < m; ++j) {
                        const double2 gdj = gd[j];
                        if (gdj.x == gdk.x) continue;
                        const bool up = gdk.x > gdj.x;
                        const double w = fabs(gdk.x - gdj.x) * fabs(gdk.y - gdj.y);
                        const double rho = 1.0 / (1.0 + exp(up ? sk - s[j] : s[j] - sk));
                        G += up ? -rho * w : rho * w;
                        H += rho * (1.0 - rho) * w;
                    }
                }
                G /= max_dcg; H /= max_dcg;
            }
            g[q0 + k] = (float)G;
            h[q0 + k] = (float)H;
        }
    }
}

int launch_lambdarank_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n, int group,
                                float* g, float* h) {
    if (n <= 0) return QGBDT_OK;
    const int64_t n_queries = (n + group - 1) / group;
    const int blocks = (int)(n_queries < 65536 ? n_queries : 65536);
    hipLaunchKernelGGL(lambdarank_grad_kernel, dim3(blocks), dim3(128), sizeof(double) * 6 * (size_t)group, ctx->stream,
                       score, label, n, group, g, h);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

int launch_logistic_gradients(qgbdt_ctx* ctx, const float* score, const float* label, int64_t n, float* g, float* h) {
    if (n <= 0) return QGBDT_OK;
    const bool vec = ((((uintptr_t)score | (uintptr_t)label | (uintptr_t)g | (uintptr_t)h) & 15) == 0);
    int blocks = (int)(((vec ? (n + 3) / 4 : n) + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (vec) hipLaunchKernelGGL(logistic_grad_kernel<true>, dim3(blocks), dim3(256), 0, ctx->stream, score, label, n, g, h);
    else hipLaunchKernelGGL(logistic_grad_kernel<false>, dim3(blocks), dim3(256), 0, ctx->stream, score, label, n, g, h);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

int launch_update_scores(qgbdt_ctx* ctx, float* score, const int32_t* row_idx, const int64_t* leaf_begin,
                         const int64_t* leaf_count, const double* leaf_value, int n_leaves,
                         const int32_t* n_leaves_dev, double lr) {
    if (n_leaves <= 0) return QGBDT_OK;
    hipLaunchKernelGGL(update_scores_kernel, dim3(REFIT_PARTS, n_leaves), dim3(256), 0, ctx->stream, score, row_idx,
                       leaf_begin, leaf_count, leaf_value, n_leaves_dev, lr);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

}  // namespace qgbdt
