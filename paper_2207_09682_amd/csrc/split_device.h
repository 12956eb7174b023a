// Device helpers of the split search shared by the stand-alone entry point and
// the tree-growing kernels.
#pragma once
#include "common.h"

namespace qgbdt {

// One histogram to scan: where it lives, whether it is first formed as
// parent - child (sibling subtraction), the totals of its leaf and where the
// best split goes.
struct ScanItem {
    int32_t slot;        // histogram index relative to the base pointer
    int32_t sub_parent;  // >= 0: hist[slot] = hist[sub_parent] - hist[sub_child] first
    int32_t sub_child;
    int32_t valid;       // 0: skip
    qgbdt_leafstat stat;
    qgbdt_split* out;
};

__device__ __forceinline__ int64_t packed_g(int64_t w) { return w >> 32; }
__device__ __forceinline__ int64_t packed_h(int64_t w) { return w & 0xffffffffLL; }

// (G*dg)^2 / (2*H*dh), fp64, this operation order (Sec. 4.1 eq. (gain)); the
// translation unit is compiled without FMA contraction.
__device__ __forceinline__ double half_loss(int64_t G, int64_t H, double dg, double dh) {
    const double a = (double)G * dg;
    const double num = a * a;
    const double den = 2.0 * ((double)H * dh);
    return num / den;
}

// Left row count from the hessian share, rounded half up, exact integers.
__device__ __forceinline__ int64_t count_estimate(int64_t HL, int64_t Hs, int64_t n) {
    return (2 * HL * n + Hs) / (2 * Hs);
}

// Reduces the per-feature candidates of one leaf to its best split: largest gain,
// ties to the lowest feature.  Called by all 64 lanes of one wavefront; lane 0
// writes the result.
__device__ inline void reduce_features_wave(const FeatCand* cand, int F, const qgbdt_leafstat& st, qgbdt_split* out,
                                            int lane) {
    double bg = 0.0;
    int bf = -1;
    for (int f = lane; f < F; f += 64) {
        const FeatCand c = cand[f];
        if (c.bin >= 0 && (c.gain > bg)) { bg = c.gain; bf = f; }  // ascending f: strict > keeps the lowest
    }
    for (int o = 32; o > 0; o >>= 1) {
        const double og = __shfl_xor(bg, o);
        const int of = __shfl_xor(bf, o);
        if (of >= 0 && (bf < 0 || og > bg || (og == bg && of < bf))) { bg = og; bf = of; }
    }
    if (lane == 0) {
        qgbdt_split s;
        s.gain = 0.0; s.feature = -1; s.bin = -1;
        s.left_g = s.left_h = s.right_g = s.right_h = s.left_count = 0;
        if (bf >= 0) {
            const FeatCand c = cand[bf];
            s.gain = c.gain; s.feature = bf; s.bin = c.bin;
            s.left_g = packed_g(c.left); s.left_h = packed_h(c.left);
            s.right_g = st.sum_g - s.left_g; s.right_h = st.sum_h - s.left_h;
            s.left_count = count_estimate(s.left_h, st.sum_h, st.n_rows);
        }
        *out = s;
    }
}

// The same reduction by a group of `sub` consecutive lanes (a power of two, 64 at most; `sl` = lane inside
// the group), so that one wavefront serves 64 / sub leaves at a time.  The winner's candidate travels with
// the comparison: no load depends on another.  Every lane of the group returns the winner's gain and feature
// (feature < 0: no split).
__device__ inline void reduce_features_lanes(const FeatCand* cand, int F, const qgbdt_leafstat& st, qgbdt_split* out,
                                             int sl, int sub, double& gain, int& feature) {
    double bg = 0.0;
    int bf = -1, bb = -1;
    int64_t bl = 0;
    for (int f0 = sl; f0 < F; f0 += 4 * sub) {  // four loads in flight
        FeatCand c[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) c[u] = cand[min(f0 + u * sub, F - 1)];
#pragma unroll
        for (int u = 0; u < 4; ++u) {  // ascending features: strict > keeps the lowest
            const int f = f0 + u * sub;
            if (f < F && c[u].bin >= 0 && (c[u].gain > bg)) { bg = c[u].gain; bf = f; bb = c[u].bin; bl = c[u].left; }
        }
    }
    for (int o = sub >> 1; o > 0; o >>= 1) {
        const double og = __shfl_xor(bg, o);
        const int of = __shfl_xor(bf, o);
        const int ob = __shfl_xor(bb, o);
        const int64_t ol = __shfl_xor(bl, o);
        if (of >= 0 && (bf < 0 || og > bg || (og == bg && of < bf))) { bg = og; bf = of; bb = ob; bl = ol; }
    }
    if (sl == 0) {
        qgbdt_split s;
        s.gain = 0.0; s.feature = -1; s.bin = -1;
        s.left_g = s.left_h = s.right_g = s.right_h = s.left_count = 0;
        if (bf >= 0) {
            s.gain = bg; s.feature = bf; s.bin = bb;
            s.left_g = packed_g(bl); s.left_h = packed_h(bl);
            s.right_g = st.sum_g - s.left_g; s.right_h = st.sum_h - s.left_h;
            s.left_count = count_estimate(s.left_h, st.sum_h, st.n_rows);
        }
        *out = s;
    }
    gain = bg;  // (all lanes of the group hold the winner)
    feature = bf;
}

}  // namespace qgbdt
