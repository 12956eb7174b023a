// Leaf-value refit with the original FP gradients (Sec. 3 eq. (leaf), Sec. 4.2):
// one gather pass over g, h through the leaf-ordered row list, fp64 sums in a
// fixed reduction order (so repeated runs give identical bits).
#include "common.h"

namespace qgbdt {

// PAIR: (g, h) of a row are read as one 8-byte pair from an interleaved copy (half the sectors
// of two separate 4-byte gathers).
template <bool PAIR>
__global__ __launch_bounds__(256) void refit_partial_kernel(const float* __restrict__ g, const float* __restrict__ h,
                                                            const float2* __restrict__ pairs,
                                                            const int32_t* __restrict__ row_idx,
                                                            const int64_t* __restrict__ leaf_begin,
                                                            const int64_t* __restrict__ leaf_count,
                                                            const int32_t* __restrict__ n_leaves_dev,
                                                            double* __restrict__ partial) {
    const int l = blockIdx.y;
    if (n_leaves_dev && l >= *n_leaves_dev) return;
    const int64_t begin = leaf_begin[l], count = leaf_count[l];
    const int64_t a = count * blockIdx.x / gridDim.x, b = count * (blockIdx.x + 1) / gridDim.x;
    double G = 0.0, H = 0.0;
    for (int64_t j = a + threadIdx.x; j < b; j += blockDim.x) {
        const int64_t i = row_idx[begin + j];
        if (PAIR) {
            const float2 v = pairs[i];
            G += (double)v.x;
            H += (double)v.y;
        } else {
            G += (double)g[i];
            H += (double)h[i];
        }
    }
    for (int o = 32; o > 0; o >>= 1) { G += __shfl_xor(G, o); H += __shfl_xor(H, o); }
    __shared__ double sg[4], sh[4];
    if ((threadIdx.x & 63) == 0) { sg[threadIdx.x >> 6] = G; sh[threadIdx.x >> 6] = H; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double* out = partial + ((int64_t)l * gridDim.x + blockIdx.x) * 2;
        out[0] = ((sg[0] + sg[1]) + sg[2]) + sg[3];
        out[1] = ((sh[0] + sh[1]) + sh[2]) + sh[3];
    }
}

__global__ void refit_final_kernel(const double* __restrict__ partial, int parts, int n_leaves,
                                   const int32_t* __restrict__ n_leaves_dev, double* __restrict__ value) {
    const int l = blockIdx.x * blockDim.x + threadIdx.x;
    if (l >= n_leaves) return;
    if (n_leaves_dev && l >= *n_leaves_dev) { value[l] = 0.0; return; }
    double G = 0.0, H = 0.0;
    for (int k = 0; k < parts; ++k) {
        G += partial[((int64_t)l * parts + k) * 2];
        H += partial[((int64_t)l * parts + k) * 2 + 1];
    }
    value[l] = (H > 0.0) ? -G / H : 0.0;
}

int launch_refit(qgbdt_ctx* ctx, const float* g, const float* h, const float2* pairs, const int32_t* row_idx,
                 const int64_t* leaf_begin, const int64_t* leaf_count, int n_leaves,
                 const int32_t* n_leaves_dev, double* value_out) {
    if (n_leaves <= 0) return QGBDT_OK;
    if (pairs)
        hipLaunchKernelGGL(refit_partial_kernel<true>, dim3(REFIT_PARTS, n_leaves), dim3(256), 0, ctx->stream, g, h,
                           pairs, row_idx, leaf_begin, leaf_count, n_leaves_dev, ctx->refit_partial);
    else
        hipLaunchKernelGGL(refit_partial_kernel<false>, dim3(REFIT_PARTS, n_leaves), dim3(256), 0, ctx->stream, g, h,
                           pairs, row_idx, leaf_begin, leaf_count, n_leaves_dev, ctx->refit_partial);
    hipLaunchKernelGGL(refit_final_kernel, dim3((n_leaves + 63) / 64), dim3(64), 0, ctx->stream, ctx->refit_partial,
                       REFIT_PARTS, n_leaves, n_leaves_dev, value_out);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

}  // namespace qgbdt
