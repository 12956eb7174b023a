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

// max|g| and max(h, 0) over all rows: every workgroup writes its pair of maxima, the
// quantizer's workgroups reduce those (atomics on one address cost ~20 ns each at the
// memory side, more than the whole stream for a few thousand workgroups).
// VEC: four rows per thread and step through 16-byte loads (g, h 16-byte aligned);
// the last n % 4 rows are taken one by one.
template <bool VEC>
__global__ __launch_bounds__(256) void absmax_kernel(const float* __restrict__ g, const float* __restrict__ h,
                                                     int64_t n, float* __restrict__ part /*[gridDim.x][2]*/) {
    float mg = 0.0f, mh = 0.0f;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (VEC) {
        const int64_t n4 = n >> 2;
        const float4* g4 = reinterpret_cast<const float4*>(g);
        const float4* h4 = reinterpret_cast<const float4*>(h);
        int64_t i = t0;
        for (; i + stride < n4; i += 2 * stride) {  // two independent steps in flight
            const float4 a = g4[i], b = h4[i], c = g4[i + stride], d = h4[i + stride];
            mg = fmaxf(mg, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
            mg = fmaxf(mg, fmaxf(fmaxf(fabsf(c.x), fabsf(c.y)), fmaxf(fabsf(c.z), fabsf(c.w))));
            mh = fmaxf(mh, fmaxf(fmaxf(b.x, b.y), fmaxf(b.z, b.w)));
            mh = fmaxf(mh, fmaxf(fmaxf(d.x, d.y), fmaxf(d.z, d.w)));
        }
        if (i < n4) {
            const float4 a = g4[i], b = h4[i];
            mg = fmaxf(mg, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
            mh = fmaxf(mh, fmaxf(fmaxf(b.x, b.y), fmaxf(b.z, b.w)));
        }
        const int64_t r = (n4 << 2) + t0;
        if (r < n) { mg = fmaxf(mg, fabsf(g[r])); mh = fmaxf(mh, h[r]); }
    } else {
        for (int64_t i = t0; i < n; i += stride) {
            mg = fmaxf(mg, fabsf(g[i]));
            mh = fmaxf(mh, h[i]);
        }
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
        part[2 * blockIdx.x] = mg;
        part[2 * blockIdx.x + 1] = mh;
    }
}

// Maxima over the partial maxima of absmax_kernel, by every thread of a 256-thread workgroup.
__device__ __forceinline__ void reduce_absmax(const float* __restrict__ part, int n_part, float& mg, float& mh) {
    mg = 0.0f; mh = 0.0f;
    for (int i = threadIdx.x; i < n_part; i += blockDim.x) {
        mg = fmaxf(mg, part[2 * i]);
        mh = fmaxf(mh, part[2 * i + 1]);
    }
    for (int o = 32; o > 0; o >>= 1) {
        mg = fmaxf(mg, __shfl_xor(mg, o));
        mh = fmaxf(mh, __shfl_xor(mh, o));
    }
    __shared__ float rg[4], rh[4];
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) { rg[w] = mg; rh[w] = mh; }
    __syncthreads();
    mg = fmaxf(fmaxf(rg[0], rg[1]), fmaxf(rg[2], rg[3]));
    mh = fmaxf(fmaxf(rh[0], rh[1]), fmaxf(rh[2], rh[3]));
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

// One row: both rounding draws come from the row's own Philox block.
__device__ __forceinline__ int quantize_row(float gv, float hv, int64_t row, float dg, float dh, int kg, int kh,
                                            uint32_t seed_lo, uint32_t seed_hi, uint32_t iteration, int rounding,
                                            int64_t& sg, int64_t& sh, int64_t& sa) {
    uint32_t r0 = 0, r1 = 0;
    if (rounding == QGBDT_ROUND_STOCHASTIC)
        philox4x32_10((uint32_t)row, (uint32_t)((uint64_t)row >> 32), iteration, 0u, seed_lo, seed_hi, r0, r1);
    const int qg = round_one(gv, dg, -kg, kg, r0, rounding);
    const int qh = kh > 0 ? round_one(hv, dh, 0, kh, r1, rounding) : (dh > 0.0f ? 1 : 0);
    sg += qg; sh += qh; sa += abs(qg);
    return ((qg << 8) | qh) & 0xffff;
}

template <bool VEC>
__global__ __launch_bounds__(256) void quantize_kernel(const float* __restrict__ g, const float* __restrict__ h,
                                                       int64_t n, const float* __restrict__ absmax_part,
                                                       int n_part, int kg, int kh, uint32_t seed_lo,
                                                       uint32_t seed_hi, uint32_t iteration, int rounding,
                                                       int16_t* __restrict__ gh, float* delta_out,
                                                       int64_t* __restrict__ totals_part /*[gridDim.x][3]*/,
                                                       float2* __restrict__ pairs /*[n] (g, h) interleaved, or null*/) {
    float mg, mh;
    reduce_absmax(absmax_part, n_part, mg, mh);
    const float dg = mg / (float)kg;
    const float dh = kh > 0 ? mh / (float)kh : mh;
    if (blockIdx.x == 0 && threadIdx.x == 0) { delta_out[0] = dg; delta_out[1] = dh; }
    int64_t sg = 0, sh = 0, sa = 0;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    const int64_t t0 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (VEC) {  // g, h 16-byte aligned, gh 8-byte aligned: four rows per thread and step
        const int64_t n4 = n >> 2;
        const float4* g4 = reinterpret_cast<const float4*>(g);
        const float4* h4 = reinterpret_cast<const float4*>(h);
        uint2* o4 = reinterpret_cast<uint2*>(gh);
        for (int64_t i = t0; i < n4; i += stride) {
            const float4 a = g4[i], b = h4[i];
            const int64_t r = i << 2;
#define QG_Q(gv, hv, k) (uint32_t)quantize_row(gv, hv, r + k, dg, dh, kg, kh, seed_lo, seed_hi, iteration, rounding, sg, sh, sa)
            const uint32_t q0 = QG_Q(a.x, b.x, 0), q1 = QG_Q(a.y, b.y, 1), q2 = QG_Q(a.z, b.z, 2), q3 = QG_Q(a.w, b.w, 3);
#undef QG_Q
            o4[i] = make_uint2(q0 | (q1 << 16), q2 | (q3 << 16));
            if (pairs) {
                float4* p4 = reinterpret_cast<float4*>(pairs + r);
                p4[0] = make_float4(a.x, b.x, a.y, b.y);
                p4[1] = make_float4(a.z, b.z, a.w, b.w);
            }
        }
        const int64_t r = (n4 << 2) + t0;
        if (r < n) {
            gh[r] = (int16_t)quantize_row(g[r], h[r], r, dg, dh, kg, kh, seed_lo, seed_hi, iteration, rounding, sg, sh, sa);
            if (pairs) pairs[r] = make_float2(g[r], h[r]);
        }
    } else {
        for (int64_t i = t0; i < n; i += stride) {
            gh[i] = (int16_t)quantize_row(g[i], h[i], i, dg, dh, kg, kh, seed_lo, seed_hi, iteration, rounding, sg, sh, sa);
            if (pairs) pairs[i] = make_float2(g[i], h[i]);
        }
    }
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
        totals_part[3 * blockIdx.x] = sg; totals_part[3 * blockIdx.x + 1] = sh; totals_part[3 * blockIdx.x + 2] = sa;
    }
}

// Sums the workgroups' partial totals: sum g~, sum h~, sum |g~|.
__global__ __launch_bounds__(256) void quantize_totals_kernel(const int64_t* __restrict__ part, int n_part,
                                                              int64_t* totals) {
    int64_t s[3] = {0, 0, 0};
    for (int i = threadIdx.x; i < n_part; i += blockDim.x)
        for (int k = 0; k < 3; ++k) s[k] += part[3 * i + k];
    __shared__ int64_t t[3][4];
    for (int k = 0; k < 3; ++k) {
        for (int o = 32; o > 0; o >>= 1) s[k] += __shfl_xor(s[k], o);
        if ((threadIdx.x & 63) == 0) t[k][threadIdx.x >> 6] = s[k];
    }
    __syncthreads();
    if (threadIdx.x < 3) totals[threadIdx.x] = t[threadIdx.x][0] + t[threadIdx.x][1] + t[threadIdx.x][2] + t[threadIdx.x][3];
}

int launch_quantize(qgbdt_ctx* ctx, const float* g, const float* h, int64_t n, int bits_g, int bits_h,
                    uint64_t seed, uint32_t iteration, int rounding, int16_t* gh, float* delta_out,
                    int64_t* totals_out, float2* pairs_out) {
    // bits_h == 0: constant hessians are not quantized (kh = 0 tells the kernel: h~ = 1, delta_h = max h)
    const int kg = (1 << (bits_g - 1)) - 1, kh = bits_h == 0 ? 0 : (1 << bits_h) - 2;
    int64_t* totals = totals_out ? totals_out : ctx->qtotals;
    const bool vec = (((uintptr_t)g | (uintptr_t)h) & 15) == 0 && ((uintptr_t)gh & 7) == 0;
    int blocks = (int)(((vec ? (n + 3) / 4 : n) + 255) / 256);
    if (blocks > QUANT_PARTS) blocks = QUANT_PARTS;
    if (blocks < 1) blocks = 1;
    if (vec) {
        hipLaunchKernelGGL(absmax_kernel<true>, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax_part);
        hipLaunchKernelGGL(quantize_kernel<true>, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax_part,
                           blocks, kg, kh, (uint32_t)seed, (uint32_t)(seed >> 32), iteration, rounding, gh, delta_out,
                           ctx->qtotals_part, pairs_out);
    } else {
        hipLaunchKernelGGL(absmax_kernel<false>, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax_part);
        hipLaunchKernelGGL(quantize_kernel<false>, dim3(blocks), dim3(256), 0, ctx->stream, g, h, n, ctx->absmax_part,
                           blocks, kg, kh, (uint32_t)seed, (uint32_t)(seed >> 32), iteration, rounding, gh, delta_out,
                           ctx->qtotals_part, pairs_out);
    }
    hipLaunchKernelGGL(quantize_totals_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->qtotals_part, blocks, totals);
    QG_HIP(ctx, hipGetLastError());
    return QGBDT_OK;
}

}  // namespace qgbdt
