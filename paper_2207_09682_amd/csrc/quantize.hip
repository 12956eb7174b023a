// Gradient quantization: interval lengths (Sec. 4.1) and stochastic / nearest
// rounding (Sec. 4.2) of per-row gradients and hessians, fp32 arithmetic.
// HBM-bound streaming kernels: 8 B read + 2 B written per row.
#include "common.h"

namespace qgbdt {

// Philox-4x32-10 (Salmon et al., SC'11): 10 rounds of two 32x32->64 multiplies
// with the Weyl key schedule.  key = seed, counter = (row lo, row hi, iteration, 0).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t& o0, uint32_t& o1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    o0 = c0; o1 = c1;
}

__global__ void absmax_init_kernel(uint32_t* absmax, int64_t* totals) {
    if (threadIdx.x < 2) absmax[threadIdx.x] = 0u;
    if (threadIdx.x < 3) totals[threadIdx.x] = 0;
}

// max|g| and max(h, 0) over all rows.  Non-negative floats order like their bit
// patterns, so the grid-wide maximum is one unsigned atomicMax per workgroup.
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ g, const float* __restrict__ h,
                                                     int64_t n, uint32_t* absmax) {
    float mg = 0.0f, mh = 0.0f;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        mg = fmaxf(mg, fabsf(g[i]));
        mh = fmaxf(mh, h[i]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        mg = fmaxf(mg, __shfl_xor(mg, o));
        mh = fmaxf(mh, __shfl_xor(mh, o));
    }
    __shared__ float sg[4], sh[4];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { sg[w] = mg; sh[w] = mh; }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int k = 1; k < 4; ++k) { mg = fmaxf(mg, sg[k]); mh = fmaxf(mh, sh[k]); }
        atomicMax(&absmax[0], __float_as_uint(mg));
        atomicMax(&absmax[1], __float_as_uint(mh));
    }
}

__device__ __forceinline__ int round_one(float v, float d, int lo, int hi, uint32_t rnd, int rounding) {
    if (!(d > 0.0f)) return 0;
    const float x = v / d;  // IEEE fp32 division
    const float fl = floorf(x);
    const float frac = x - fl;
    int up;
    if (rounding == QGBDT_ROUND_STOCHASTIC) {
        const float u = (float)(rnd >> 8) * (1.0f / 16777216.0f);
        up = (u < frac) ? 1 : 0;
    } else {
        up = (frac >= 0.5f) ? 1 : 0;
    }
    int q = (int)fl + up;
    return min(max(q, lo), hi);
}

__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ g, const float* __restrict__ h,
                                                       int64_t n, const uint32_t* __restrict__ absmax, int kg,
                                                       int kh, uint32_t seed_lo, uint32_t seed_hi,
                                                       uint32_t iteration, int rounding,
                                                       int16_t* __restrict__ gh, float* delta_out,
                                                       int64_t* totals) {
    const float dg = __uint_as_float(absmax[0]) / (float)kg;
    const float dh = __uint_as_float(absmax[1]) / (float)kh;
    if (blockIdx.x == 0 && threadIdx.x == 0) { delta_out[0] = dg; delta_out[1] = dh; }
    int64_t sg = 0, sh = 0, sa = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
        uint32_t r0 = 0, r1 = 0;
        if (rounding == QGBDT_ROUND_STOCHASTIC)
            philox4x32_10((uint32_t)i, (uint32_t)((uint64_t)i >> 32), iteration, 0u, seed_lo, seed_hi, r0, r1);
        const int qg = round_one(g[i], dg, -kg, kg, r0, rounding);
        const int qh = round_one(h[i], dh, 0, kh, r1, rounding);
        gh[i] = (int16_t)((qg << 8) | qh);
        sg += qg; sh += qh; sa += abs(qg);
    }
    if (totals) {
        for (int o = 32; o > 0; o >>= 1) {
            sg += __shfl_xor(sg, o);
            sh += __shfl_xor(sh, o);
            sa += __shfl_xor(sa, o);
        }
        __shared__ int64_t tg[4], th[4], ta[4];
        const int w = threadIdx.x >> 6;
        if ((threadIdx.x & 63) == 0) { tg[w] = sg; th[w] = sh; ta[w] = sa; }
        __syncthreads();
        if (threadIdx.x == 0) {
            for (int k = 1; k < 4; ++k) { sg += tg[k]; sh += th[k]; sa += ta[k]; }
            atomicAdd((unsigned long long*)&totals[0], (unsigned long long)sg);
            atomicAdd((unsigned long long*)&totals[1], (unsigned long long)sh);
            atomicAdd((unsigned long long*)&totals[2], (unsigned long long)sa);
        }
    }
}

int launch_quantize(qgbdt_ctx* ctx, const float* g, const float* h, int64_t n, int bits_g, int bits_h,
                    uint64_t seed, uint32_t iteration, int rounding, int16_t* gh, float* delta_out,
                    int64_t* totals_out) {
    const int kg = (1 << (bits_g - 1)) - 1, kh = (1 << bits_h) - 2;
    int64_t* totals = totals_out ? totals_out : ctx->qtotals;
    hipLaunchKernelGGL(absmax_init_kernel, dim3(1), dim3(64), 0, ctx->stream, ctx->absmax, totals);
    int blocks = (int)((n + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(absmax_kernel, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax);
    hipLaunchKernelGGL(quantize_kernel, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax, kg, kh,
                       (uint32_t)seed, (uint32_t)(seed >> 32), iteration, rounding, gh, delta_out, totals);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

}  // namespace qgbdt
