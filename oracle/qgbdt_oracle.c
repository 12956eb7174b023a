/*
 * qgbdt_oracle.c -- CPU oracle for the quantized-GBDT hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
 * GPU library must compute.  It is used by the tests, by the smoke check and by
 * the benchmark's CPU-baseline leg, never by the product path.  It shares no
 * code, header, table or constant generator with the HIP sources.
 *
 * Arithmetic: every integer sum is int64 (so a narrow-accumulator overflow on
 * the GPU shows up as a mismatch), gains and leaf values are fp64, the
 * quantizer works in fp32 as stated below.  No blocking, fusion or reordering
 * beyond what each passage states.  Build with -ffp-contract=off.
 *
 * Passages followed (arxiv 2207.09682):
 *   scales            Sec. 4.1, first display equation (delta_g, delta_h)
 *   quantize          Sec. 4.1 eq. (scale); Sec. 4.2 definitions of RN and SR
 *   histogram         Algorithm 1 with g~, h~ substituted (Sec. 4.1)
 *   split gain        Sec. 4.1 eq. (gain); enumeration per Sec. 3
 *   leaf value        Sec. 3 eq. (leaf); refit per Sec. 4.2
 *   packed word       Sec. 6.2
 *   width rule        Sec. 7.4.3 (minimum width with no overflow)
 *   growth            Sec. 3 (greedy splitting) and Sec. 7 (leaf-wise)
 *   loss derivatives  Sec. 3 (g_i, h_i of the loss; binary cross-entropy), score update Sec. 3
 * The random numbers of stochastic rounding come from Philox-4x32-10 (Salmon et
 * al., "Parallel random numbers: as easy as 1, 2, 3", SC'11), written here from
 * that paper's description; it is pinned by the published known-answer vectors.
 *
 * Pins: see tests/test_oracle_*.py.  Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define QREF_OK 0
#define QREF_E_ARG (-1)
#define QREF_E_ALLOC (-2)
#define QREF_E_SIBLING (-3)
#define QREF_E_RANGE (-4)

/* ------------------------------------------------------------------------ */
/* Philox-4x32-10                                                            */
/* ------------------------------------------------------------------------ */

static void philox_round(uint32_t c[4], const uint32_t k[2]) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c[2];
    const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
    const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
    const uint32_t n0 = hi1 ^ c[1] ^ k[0];
    const uint32_t n1 = lo1;
    const uint32_t n2 = hi0 ^ c[3] ^ k[1];
    const uint32_t n3 = lo0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

void qgbdt_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c[4] = {ctr[0], ctr[1], ctr[2], ctr[3]};
    uint32_t k[2] = {key[0], key[1]};
    for (int r = 0; r < 10; ++r) {
        if (r > 0) { k[0] += 0x9E3779B9u; k[1] += 0xBB67AE85u; }
        philox_round(c, k);
    }
    out[0] = c[0]; out[1] = c[1]; out[2] = c[2]; out[3] = c[3];
}

/* Uniform in [0,1) with 24 bits, exact in fp32.
 * key = seed (low word, high word); counter = (row low, row high, iteration, 0).
 * stream 0 (gradient) takes output word 0, stream 1 (hessian) output word 1, so
 * the two roundings of one row are independent (the proofs in App. B assume it). */
float qgbdt_ref_uniform24(uint64_t seed, uint32_t iteration, uint64_t row, int stream) {
    uint32_t ctr[4] = {(uint32_t)row, (uint32_t)(row >> 32), iteration, 0u};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    qgbdt_ref_philox4x32_10(ctr, key, out);
    return (float)(out[stream & 1] >> 8) * (1.0f / 16777216.0f);
}

/* ------------------------------------------------------------------------ */
/* Scales and quantizer (Sec. 4.1, Sec. 4.2)                                  */
/* ------------------------------------------------------------------------ */

static int level_g(int bits) { return (1 << (bits - 1)) - 1; } /* 2^(B-1) - 1 */
static int level_h(int bits) { return bits == 0 ? 1 : (1 << bits) - 2; } /* 2^B - 2; 1 when h is not quantized */

/* delta[0] = max|g| / (2^(B_g-1)-1), delta[1] = max(h) / (2^B_h - 2), fp32 division.
 * The maximum runs over all n rows.  max(h) is taken as 0 when every h is negative. */
int qgbdt_ref_scales(const float* g, const float* h, int64_t n, int bits_g, int bits_h,
                     float* delta) {
    if (bits_g < 2 || bits_g > 8 || !(bits_h == 0 || (bits_h >= 2 && bits_h <= 8)) || n < 0) return QREF_E_ARG;
    float mg = 0.0f, mh = 0.0f;
    for (int64_t i = 0; i < n; ++i) {
        const float a = fabsf(g[i]);
        if (a > mg) mg = a;
        if (h[i] > mh) mh = h[i];
    }
    delta[0] = mg / (float)level_g(bits_g);
    /* bits_h == 0: the hessians are one constant and are not quantized (Sec. 4.1, remark after
     * eq. (scale)): every h~_i is 1 and delta_h is the constant itself */
    delta[1] = (bits_h == 0) ? mh : mh / (float)level_h(bits_h);
    return QREF_OK;
}

/* Round(v / d) clamped to [lo, hi].  rounding 0 = SR with uniform u, 1 = RN.
 * d == 0 (all values zero) maps everything to 0. */
static int round_one(float v, float d, int lo, int hi, float u, int rounding) {
    if (!(d > 0.0f)) return 0;
    const float x = v / d;
    const float fl = floorf(x);
    const float frac = x - fl; /* exact: |x| is far below 2^23 */
    int up;
    if (rounding == 0) up = (u < frac) ? 1 : 0;      /* ceil w.p. x - floor(x) */
    else up = (frac >= 0.5f) ? 1 : 0;                /* RN: half goes up        */
    int q = (int)fl + up;
    if (q < lo) q = lo;
    if (q > hi) q = hi;
    return q;
}

int qgbdt_ref_quantize_gradients(const float* g, const float* h, int64_t n, int bits_g,
                                 int bits_h, uint64_t seed, uint32_t iteration, int rounding,
                                 int8_t* gq, uint8_t* hq, float* delta) {
    int rc = qgbdt_ref_scales(g, h, n, bits_g, bits_h, delta);
    if (rc != QREF_OK) return rc;
    if (rounding != 0 && rounding != 1) return QREF_E_ARG;
    const int kg = level_g(bits_g), kh = level_h(bits_h);
    for (int64_t i = 0; i < n; ++i) {
        float ug = 0.0f, uh = 0.0f;
        if (rounding == 0) {
            ug = qgbdt_ref_uniform24(seed, iteration, (uint64_t)i, 0);
            uh = qgbdt_ref_uniform24(seed, iteration, (uint64_t)i, 1);
        }
        gq[i] = (int8_t)round_one(g[i], delta[0], -kg, kg, ug, rounding);
        hq[i] = (bits_h == 0) ? (uint8_t)(delta[1] > 0.0f ? 1 : 0)
                              : (uint8_t)round_one(h[i], delta[1], 0, kh, uh, rounding);
    }
    return QREF_OK;
}

/* ------------------------------------------------------------------------ */
/* Packed words (Sec. 6.2) and the width rule (Sec. 7.4.3)                    */
/* ------------------------------------------------------------------------ */

/* word = G * 2^w + H, gradient in the upper (signed) half, hessian in the lower
 * half read as unsigned.  w = 16 gives a 32-bit word, w = 32 a 64-bit word; the
 * result is returned sign-extended in an int64.  Returns QREF_E_RANGE when a
 * field does not fit. */
int qgbdt_ref_pack(int64_t G, int64_t H, int w, int64_t* word) {
    if (w != 16 && w != 32) return QREF_E_ARG;
    const int64_t gmax = ((int64_t)1 << (w - 1)) - 1, gmin = -gmax - 1;
    const int64_t hmax = ((int64_t)1 << w) - 1;
    if (G < gmin || G > gmax || H < 0 || H > hmax) return QREF_E_RANGE;
    *word = G * ((int64_t)1 << w) + H;
    return QREF_OK;
}

void qgbdt_ref_unpack(int64_t word, int w, int64_t* G, int64_t* H) {
    const int64_t m = ((int64_t)1 << w);
    int64_t lo = word % m;
    if (lo < 0) lo += m;
    *H = lo;
    *G = (word - lo) / m;
}

/* Largest number of rows whose sums are guaranteed to fit fields of width w:
 * n*k_g <= 2^(w-1)-1 and n*k_h <= 2^w-1. */
int64_t qgbdt_ref_max_rows_for_width(int bits_g, int bits_h, int w) {
    const int64_t kg = level_g(bits_g), kh = level_h(bits_h);
    const int64_t a = ((((int64_t)1) << (w - 1)) - 1) / kg;
    const int64_t b = ((((int64_t)1) << w) - 1) / kh;
    return a < b ? a : b;
}

/* ------------------------------------------------------------------------ */
/* Histogram (Algorithm 1 with g~, h~)                                        */
/* ------------------------------------------------------------------------ */

static inline int bin_at(const void* bins, int bin_bytes, int64_t row, int F, int f) {
    if (bin_bytes == 1) return ((const uint8_t*)bins)[row * F + f];
    return ((const uint16_t*)bins)[row * F + f];
}

/* hist[(f*nb + b)*2 + 0] = sum of g~, [...+1] = sum of h~ over the leaf's rows.
 * Rows are row_idx[begin .. begin+count) or, if row_idx is NULL, begin .. begin+count. */
int qgbdt_ref_build_histograms(const void* bins, int bin_bytes, int F, int nb,
                               const int8_t* gq, const uint8_t* hq, const int32_t* row_idx,
                               int64_t begin, int64_t count, int64_t* hist) {
    if ((bin_bytes != 1 && bin_bytes != 2) || F <= 0 || nb <= 0 || count < 0) return QREF_E_ARG;
    memset(hist, 0, sizeof(int64_t) * 2 * (size_t)F * (size_t)nb);
#pragma omp parallel for schedule(static)
    for (int f = 0; f < F; ++f) {
        int64_t* hf = hist + (size_t)f * nb * 2;
        for (int64_t j = begin; j < begin + count; ++j) {
            const int64_t i = row_idx ? (int64_t)row_idx[j] : j;
            const int b = bin_at(bins, bin_bytes, i, F, f);
            hf[2 * b + 0] += gq[i];
            hf[2 * b + 1] += hq[i];
        }
    }
    return QREF_OK;
}

/* sibling = parent - child, element-wise over n_words int64 values. */
int qgbdt_ref_subtract_histograms(const int64_t* parent, const int64_t* child, int64_t* sibling,
                                  int64_t n_words) {
    for (int64_t k = 0; k < n_words; ++k) sibling[k] = parent[k] - child[k];
    return QREF_OK;
}

/* ------------------------------------------------------------------------ */
/* Best split of one leaf (Sec. 3 enumeration, Sec. 4.1 eq. (gain))           */
/* ------------------------------------------------------------------------ */

typedef struct {
    double gain;
    int32_t feature, bin;
    int64_t GL, HL, GR, HR;
    int64_t cnt_left; /* estimated from hessians */
} qref_split;

/* (G*dg)^2 / (2*H*dh) in fp64, evaluated left to right. */
static double half_loss(int64_t G, int64_t H, double dg, double dh) {
    const double a = (double)G * dg;
    const double num = a * a;
    const double den = 2.0 * ((double)H * dh);
    return num / den;
}

/* Row count of the left side estimated from the hessian share, rounded half up,
 * in exact integer arithmetic: floor((2*HL*n + Hs) / (2*Hs)). */
static int64_t count_estimate(int64_t HL, int64_t Hs, int64_t n) {
    return (2 * HL * n + Hs) / (2 * Hs);
}

/* Thresholds t = 0 .. nb-2; rows with bin <= t go left.  A candidate is valid iff
 * HL > 0, HR > 0, both estimated counts >= min_data, both H*dh >= min_sum_hess.
 * The first candidate (ascending feature, then bin) with the strictly largest
 * gain > 0 wins.  feature = -1 when there is none. */
int qgbdt_ref_find_best_split(const int64_t* hist, int F, int nb, int64_t n_rows, int64_t Gs,
                              int64_t Hs, float delta_g, float delta_h, int64_t min_data,
                              double min_sum_hess, double* gain, int32_t* feature, int32_t* bin,
                              int64_t* stats /* GL,HL,GR,HR,cntL */) {
    const double dg = (double)delta_g, dh = (double)delta_h;
    qref_split best;
    best.gain = 0.0; best.feature = -1; best.bin = -1;
    best.GL = best.HL = best.GR = best.HR = best.cnt_left = 0;
    if (Hs > 0) {
        const double parent = half_loss(Gs, Hs, dg, dh);
        for (int f = 0; f < F; ++f) {
            int64_t GL = 0, HL = 0;
            for (int t = 0; t + 1 < nb; ++t) {
                GL += hist[((size_t)f * nb + t) * 2 + 0];
                HL += hist[((size_t)f * nb + t) * 2 + 1];
                const int64_t GR = Gs - GL, HR = Hs - HL;
                if (HL <= 0 || HR <= 0) continue;
                const int64_t cl = count_estimate(HL, Hs, n_rows), cr = n_rows - cl;
                if (cl < min_data || cr < min_data) continue;
                if ((double)HL * dh < min_sum_hess || (double)HR * dh < min_sum_hess) continue;
                const double gn = half_loss(GL, HL, dg, dh) + half_loss(GR, HR, dg, dh) - parent;
                if (gn > best.gain) {
                    best.gain = gn; best.feature = f; best.bin = t;
                    best.GL = GL; best.HL = HL; best.GR = GR; best.HR = HR; best.cnt_left = cl;
                }
            }
        }
    }
    *gain = best.gain; *feature = best.feature; *bin = best.bin;
    stats[0] = best.GL; stats[1] = best.HL; stats[2] = best.GR; stats[3] = best.HR;
    stats[4] = best.cnt_left;
    return QREF_OK;
}

/* ------------------------------------------------------------------------ */
/* Row partition                                                              */
/* ------------------------------------------------------------------------ */

/* Stable: rows of row_idx[begin..begin+count) with bins[row][feature] <= bin come
 * first, in their old order, then the others in their old order. */
int qgbdt_ref_partition_rows(const void* bins, int bin_bytes, int F, int32_t* row_idx,
                             int64_t begin, int64_t count, int feature, int bin,
                             int64_t* n_left) {
    if (count < 0 || feature < 0 || feature >= F) return QREF_E_ARG;
    int32_t* right = (int32_t*)malloc(sizeof(int32_t) * (size_t)(count > 0 ? count : 1));
    if (!right) return QREF_E_ALLOC;
    int64_t nl = 0, nr = 0;
    for (int64_t j = begin; j < begin + count; ++j) {
        const int32_t i = row_idx[j];
        if (bin_at(bins, bin_bytes, i, F, feature) <= bin) row_idx[begin + nl++] = i;
        else right[nr++] = i;
    }
    memcpy(row_idx + begin + nl, right, sizeof(int32_t) * (size_t)nr);
    free(right);
    *n_left = nl;
    return QREF_OK;
}

/* ------------------------------------------------------------------------ */
/* Leaf refit (Sec. 3 eq. (leaf) with the original FP gradients, Sec. 4.2)    */
/* ------------------------------------------------------------------------ */

/* value[l] = -sum(g)/sum(h) over the leaf's rows, fp64 sums in list order; 0 when
 * sum(h) is not positive. */
int qgbdt_ref_refit_leaves(const float* g, const float* h, const int32_t* row_idx,
                           const int64_t* leaf_begin, const int64_t* leaf_count, int n_leaves,
                           double* value) {
    for (int l = 0; l < n_leaves; ++l) {
        double G = 0.0, H = 0.0;
        for (int64_t j = leaf_begin[l]; j < leaf_begin[l] + leaf_count[l]; ++j) {
            G += (double)g[row_idx[j]];
            H += (double)h[row_idx[j]];
        }
        value[l] = (H > 0.0) ? -G / H : 0.0;
    }
    return QREF_OK;
}

/* Leaf value from the quantized sums (Sec. 4.2, the expression for w~*). */
double qgbdt_ref_quantized_leaf_value(int64_t G, int64_t H, float delta_g, float delta_h) {
    if (H <= 0 || !(delta_h > 0.0f)) return 0.0;
    return -((double)G * (double)delta_g) / ((double)H * (double)delta_h);
}

/* ------------------------------------------------------------------------ */
/* Around the tree: loss derivatives and score update (Sec. 3)                */
/* ------------------------------------------------------------------------ */

/* g_i, h_i = first and second derivative of the loss w.r.t. the current prediction
 * (Sec. 3), for the binary cross-entropy loss l(s, y) = -y log p - (1-y) log(1-p),
 * p = 1 / (1 + exp(-s)):  g = p - y,  h = p (1 - p).  Evaluated in fp64 from the fp32
 * inputs and rounded once to fp32, so the values are the correctly rounded ones. */
int qgbdt_ref_logistic_gradients(const float* score, const float* label, int64_t n, float* g, float* h) {
    for (int64_t i = 0; i < n; ++i) {
        const double p = 1.0 / (1.0 + exp(-(double)score[i]));
        g[i] = (float)(p - (double)label[i]);
        h[i] = (float)(p * (1.0 - p));
    }
    return QREF_OK;
}

/* Pairwise ranking loss with NDCG weights (the lambdarank objective the paper's ranking
 * experiments name in its parameter tables; the textbook LambdaRank of Burges et al.).  Rows come
 * in consecutive queries of `group` rows (the last may be shorter); label = integer relevance.
 * Inside a query: documents are ranked by score, descending, ties by position; gain = 2^rel - 1,
 * discount(rank) = 1 / log2(rank + 2), maxDCG = DCG of the gains sorted descending.  For every
 * pair (a, b) with rel_a > rel_b:
 *     rho = 1 / (1 + exp(s_a - s_b)),  w = |gain_a - gain_b| * |disc_a - disc_b| / maxDCG,
 *     g_a -= rho w,  g_b += rho w,  h_a += rho (1 - rho) w,  h_b += rho (1 - rho) w.
 * fp64 throughout, pairs in (a ascending, b ascending) order, rounded once to fp32. */
int qgbdt_ref_lambdarank_gradients(const float* score, const float* label, int64_t n, int group,
                                   float* g, float* h) {
    if (group < 1 || n < 0) return QREF_E_ARG;
    double* G = (double*)malloc(sizeof(double) * (size_t)group);
    double* H = (double*)malloc(sizeof(double) * (size_t)group);
    double* gain = (double*)malloc(sizeof(double) * (size_t)group);
    double* disc = (double*)malloc(sizeof(double) * (size_t)group);
    if (!G || !H || !gain || !disc) { free(G); free(H); free(gain); free(disc); return QREF_E_ALLOC; }
    for (int64_t q0 = 0; q0 < n; q0 += group) {
        const int m = (int)((n - q0 < group) ? (n - q0) : group);
        const float* s = score + q0;
        const float* r = label + q0;
        double max_dcg = 0.0;
        for (int k = 0; k < m; ++k) {
            int rank = 0, irank = 0;
            gain[k] = exp2((double)r[k]) - 1.0;
            for (int j = 0; j < m; ++j) {
                if (s[j] > s[k] || (s[j] == s[k] && j < k)) ++rank;
                if (r[j] > r[k] || (r[j] == r[k] && j < k)) ++irank; /* position among the gains sorted descending */
            }
            disc[k] = 1.0 / log2((double)rank + 2.0);
            max_dcg += gain[k] / log2((double)irank + 2.0);
            G[k] = 0.0; H[k] = 0.0;
        }
        if (max_dcg > 0.0) {
            for (int a = 0; a < m; ++a)
                for (int b = 0; b < m; ++b) {
                    if (!(r[a] > r[b])) continue;
                    const double rho = 1.0 / (1.0 + exp((double)s[a] - (double)s[b]));
                    const double w = fabs(gain[a] - gain[b]) * fabs(disc[a] - disc[b]) / max_dcg;
                    G[a] -= rho * w; G[b] += rho * w;
                    H[a] += rho * (1.0 - rho) * w; H[b] += rho * (1.0 - rho) * w;
                }
        }
        for (int k = 0; k < m; ++k) { g[q0 + k] = (float)G[k]; h[q0 + k] = (float)H[k]; }
    }
    free(G); free(H); free(gain); free(disc);
    return QREF_OK;
}

/* Prediction update after a tree (Sec. 3: the tree's leaf values are added to the current
 * predictions; the learning rate scales them):  score_i += (float)(lr * value[leaf(i)]),
 * one fp32 addition per row.  Leaves are slices of the leaf-ordered row list. */
int qgbdt_ref_update_scores(float* score, const int32_t* row_idx, const int64_t* leaf_begin,
                            const int64_t* leaf_count, const double* leaf_value, int n_leaves, double lr) {
    for (int l = 0; l < n_leaves; ++l) {
        const float d = (float)(lr * leaf_value[l]);
        for (int64_t j = leaf_begin[l]; j < leaf_begin[l] + leaf_count[l]; ++j) score[row_idx[j]] += d;
    }
    return QREF_OK;
}

/* ------------------------------------------------------------------------ */
/* One tree, leaf-wise                                                        */
/* ------------------------------------------------------------------------ */

typedef struct {
    int64_t begin, count;
    int64_t G, H;
    int64_t* hist;
    qref_split best;
} qref_leaf;

static void eval_leaf(qref_leaf* lf, int F, int nb, float dg, float dh, int64_t min_data,
                      double min_sum_hess) {
    int64_t st[5];
    qgbdt_ref_find_best_split(lf->hist, F, nb, lf->count, lf->G, lf->H, dg, dh, min_data,
                              min_sum_hess, &lf->best.gain, &lf->best.feature, &lf->best.bin, st);
    lf->best.GL = st[0]; lf->best.HL = st[1]; lf->best.GR = st[2]; lf->best.HR = st[3];
    lf->best.cnt_left = st[4];
}

/*
 * Grows one tree.  Quantizes (g,h) with (seed, iteration), builds the root
 * histogram, then repeatedly splits the open leaf with the largest gain (ties:
 * lowest leaf id) until num_leaves leaves exist or no leaf has a gain > 0.  The
 * left child keeps the parent's leaf id, the right child takes the next free id.
 * After a split the child with fewer rows (tie: left) gets its histogram built
 * from its rows, the other one is parent - that; with verify_sibling != 0 the
 * other one is also built directly and compared (QREF_E_SIBLING on a mismatch).
 * Leaf values are refit from the FP gradients at the end.
 *
 * Outputs (caller-allocated):
 *   n_leaves_out[1]; split_* [num_leaves-1] in split order: the leaf split, its
 *   feature, threshold bin, gain, (GL,HL,GR,HR) quantized sums and the true left
 *   row count; leaf_* [num_leaves] by leaf id; row_idx_out[N] leaf-ordered rows;
 *   delta_out[2]; gq_out[N], hq_out[N]; hist_units_out[1] = sum over histogram
 *   builds of rows*features actually accumulated.
 */
int qgbdt_ref_grow_tree(const void* bins, int bin_bytes, int64_t N, int F, int nb, const float* g,
                        const float* h, int bits_g, int bits_h, uint64_t seed, uint32_t iteration,
                        int rounding, int num_leaves, int64_t min_data, double min_sum_hess,
                        int verify_sibling, int32_t* n_leaves_out, int32_t* split_leaf,
                        int32_t* split_feature, int32_t* split_bin, double* split_gain,
                        int64_t* split_stats /* [L-1][4] */, int64_t* split_n_left,
                        int64_t* leaf_begin, int64_t* leaf_count, int64_t* leaf_G,
                        int64_t* leaf_H, double* leaf_value, double* leaf_value_quant,
                        int32_t* row_idx_out, float* delta_out, int8_t* gq_out, uint8_t* hq_out,
                        int64_t* hist_units_out) {
    if (num_leaves < 1 || N <= 0 || N > 2147483647LL) return QREF_E_ARG;
    int rc = qgbdt_ref_quantize_gradients(g, h, N, bits_g, bits_h, seed, iteration, rounding,
                                          gq_out, hq_out, delta_out);
    if (rc != QREF_OK) return rc;
    const float dg = delta_out[0], dh = delta_out[1];
    const size_t hwords = (size_t)F * nb * 2;
    qref_leaf* leaves = (qref_leaf*)calloc((size_t)num_leaves, sizeof(qref_leaf));
    int64_t* check = verify_sibling ? (int64_t*)malloc(sizeof(int64_t) * hwords) : NULL;
    if (!leaves || (verify_sibling && !check)) { free(leaves); free(check); return QREF_E_ALLOC; }
    for (int64_t i = 0; i < N; ++i) row_idx_out[i] = (int32_t)i;
    int64_t units = 0;

    qref_leaf* root = &leaves[0];
    root->begin = 0; root->count = N;
    root->hist = (int64_t*)malloc(sizeof(int64_t) * hwords);
    if (!root->hist) { free(leaves); free(check); return QREF_E_ALLOC; }
    for (int64_t i = 0; i < N; ++i) { root->G += gq_out[i]; root->H += hq_out[i]; }
    qgbdt_ref_build_histograms(bins, bin_bytes, F, nb, gq_out, hq_out, row_idx_out, 0, N,
                               root->hist);
    units += N * (int64_t)F;
    eval_leaf(root, F, nb, dg, dh, min_data, min_sum_hess);

    int n_leaves = 1;
    rc = QREF_OK;
    while (n_leaves < num_leaves) {
        int s = -1;
        double bg = 0.0;
        for (int l = 0; l < n_leaves; ++l)
            if (leaves[l].best.feature >= 0 && leaves[l].best.gain > bg) { bg = leaves[l].best.gain; s = l; }
        if (s < 0) break;
        const int k = n_leaves - 1; /* split number */
        qref_leaf* P = &leaves[s];
        qref_leaf* R = &leaves[n_leaves];
        const qref_split sp = P->best;
        int64_t nl = 0;
        rc = qgbdt_ref_partition_rows(bins, bin_bytes, F, row_idx_out, P->begin, P->count,
                                      sp.feature, sp.bin, &nl);
        if (rc != QREF_OK) break;
        split_leaf[k] = s; split_feature[k] = sp.feature; split_bin[k] = sp.bin;
        split_gain[k] = sp.gain;
        split_stats[4 * k + 0] = sp.GL; split_stats[4 * k + 1] = sp.HL;
        split_stats[4 * k + 2] = sp.GR; split_stats[4 * k + 3] = sp.HR;
        split_n_left[k] = nl;

        int64_t* parent_hist = P->hist;
        const int64_t pbegin = P->begin, pcount = P->count;
        /* left child reuses slot s, right child is the new leaf */
        qref_leaf L;
        memset(&L, 0, sizeof(L));
        L.begin = pbegin; L.count = nl; L.G = sp.GL; L.H = sp.HL;
        R->begin = pbegin + nl; R->count = pcount - nl; R->G = sp.GR; R->H = sp.HR;
        qref_leaf* small = (L.count <= R->count) ? &L : R;
        qref_leaf* large = (small == &L) ? R : &L;
        small->hist = (int64_t*)malloc(sizeof(int64_t) * hwords);
        if (!small->hist) { rc = QREF_E_ALLOC; break; }
        qgbdt_ref_build_histograms(bins, bin_bytes, F, nb, gq_out, hq_out, row_idx_out,
                                   small->begin, small->count, small->hist);
        units += small->count * (int64_t)F;
        large->hist = parent_hist; /* parent - small, in place */
        qgbdt_ref_subtract_histograms(parent_hist, small->hist, large->hist, (int64_t)hwords);
        if (verify_sibling) {
            qgbdt_ref_build_histograms(bins, bin_bytes, F, nb, gq_out, hq_out, row_idx_out,
                                       large->begin, large->count, check);
            if (memcmp(check, large->hist, sizeof(int64_t) * hwords) != 0) { rc = QREF_E_SIBLING; }
        }
        *P = L;
        ++n_leaves;
        if (rc != QREF_OK) break;
        eval_leaf(&leaves[s], F, nb, dg, dh, min_data, min_sum_hess);
        eval_leaf(&leaves[n_leaves - 1], F, nb, dg, dh, min_data, min_sum_hess);
    }

    if (rc == QREF_OK) {
        *n_leaves_out = n_leaves;
        for (int l = 0; l < n_leaves; ++l) {
            leaf_begin[l] = leaves[l].begin; leaf_count[l] = leaves[l].count;
            leaf_G[l] = leaves[l].G; leaf_H[l] = leaves[l].H;
            leaf_value_quant[l] = qgbdt_ref_quantized_leaf_value(leaves[l].G, leaves[l].H, dg, dh);
        }
        qgbdt_ref_refit_leaves(g, h, row_idx_out, leaf_begin, leaf_count, n_leaves, leaf_value);
        *hist_units_out = units;
    }
    for (int l = 0; l < num_leaves; ++l) free(leaves[l].hist);
    free(leaves); free(check);
    return rc;
}
