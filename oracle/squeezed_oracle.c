/*
 * CPU oracle for the online path of Squeezed Attention (arxiv 2411.09688).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
 * method computes, used by the tests, the smoke check and the benchmark's CPU
 * baseline.  It shares no code, header, table or helper with the GPU library,
 * and the GPU library never calls it.
 *
 * Every function handles one problem with plain loops, one (sequence, head,
 * query) at a time, in the order and notation of the paper:
 *
 *   oracle_centroid_score   Eq. 1 (Section 3.2) in the max-subtracted form of
 *                           Appendix D "Generation Stage": x_i, m, e_i, D.
 *   oracle_select           the rule "load cluster i iff S_i > T" (Section 3.2,
 *                           Section 4.1), evaluated as e_i > T*D (Appendix D),
 *                           and the kept clusters' key ranges (the key-index
 *                           tensor of Section 4.2, as ranges because keys are
 *                           stored sorted by cluster).
 *   oracle_select_mean      the prefill rule of Appendix D "Prefill Stage": the scores
 *                           of Eq. 1 are averaged over all query tokens of a
 *                           (sequence, head) and the average is compared with T,
 *                           giving one kept set shared by the query tokens.
 *   oracle_hier_select      Eq. 2 and Eq. 3 (Section 3.3): level 1 on the coarse
 *                           centroids, level 2 on the children of the kept
 *                           coarse clusters with the normaliser over those
 *                           children only.
 *   oracle_multilevel_select  the same, level after level, for any number of
 *                           levels (Section 3.3 notes the extension).
 *   oracle_sparse_attn      exact softmax attention over the kept fixed-context
 *                           keys together with the user keys (Section 3.2,
 *                           Section 4.2), one softmax over the union.
 *
 * Precision.  Scores and the keep decision are taken in fp32 on the fp16
 * inputs, because a float comparison decides an integer result (the kept set)
 * and the GPU kernels take the same decision in fp32.  Attention, given the
 * kept set, is accumulated in fp64.
 *
 * Parity pins: see tests/test_oracle_*.py (closed forms, library softmax for
 * the C = L special case, brute force with a literal fp64 evaluation of the
 * equations, keep-all == dense attention, merge invariants).  The paper prints
 * no worked numeric example of S_i, a selection or an attention output, so no
 * value here is pinned to a number printed in the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* IEEE binary16 -> binary32, exact. */
static float h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t ex = (h >> 10) & 0x1fu;
    uint32_t man = h & 0x3ffu;
    uint32_t bits;
    if (ex == 0) {
        if (man == 0) {
            bits = sign;
        } else { /* subnormal: value = man * 2^-24 */
            float v = (float)man * 5.9604644775390625e-08f;
            memcpy(&bits, &v, 4);
            bits |= sign;
        }
    } else if (ex == 31) {
        bits = sign | 0x7f800000u | (man << 13);
    } else {
        bits = sign | ((ex + 112u) << 23) | (man << 13);
    }
    float f;
    memcpy(&f, &bits, 4);
    return f;
}

/* x_i = sm_scale * sum_u q_u C_{i,u}, u ascending, fp32 (argument of exp in Eq. 1). */
static float scaled_dot_f32(const uint16_t *a, const uint16_t *b, int d, float sm_scale)
{
    float acc = 0.0f;
    for (int u = 0; u < d; ++u)
        acc += h2f(a[u]) * h2f(b[u]);
    return sm_scale * acc;
}

/*
 * Scores of one query against a list of centroids (Eq. 1, max-subtracted).
 *   cand == NULL : centroids 0..n-1;  else centroid ids cand[0..n-1].
 * Outputs x[0..n-1] (position-indexed), *m = max x over clusters with N>0,
 * *D = sum_i N_i exp(x_i - m), i ascending.
 * Zero-size clusters hold no keys: they add nothing to D and do not set m.
 */
static void score_one(const uint16_t *q, const uint16_t *cent, const int32_t *sizes,
                      const int32_t *cand, int n, int d, float sm_scale,
                      float *x, float *m_out, float *D_out)
{
    float m = -INFINITY;
    for (int i = 0; i < n; ++i) {
        int c = cand ? cand[i] : i;
        x[i] = scaled_dot_f32(q, cent + (size_t)c * d, d, sm_scale);
        if (sizes[c] > 0 && x[i] > m)
            m = x[i];
    }
    float D = 0.0f;
    for (int i = 0; i < n; ++i) {
        int c = cand ? cand[i] : i;
        if (sizes[c] > 0)
            D += (float)sizes[c] * expf(x[i] - m);
    }
    *m_out = m;
    *D_out = D;
}

/* keep_i  <=>  N_i > 0  and  exp(x_i - m) > T * D   (strict). */
static int keep_rule(float x, float m, float D, float T, int32_t N)
{
    return N > 0 && expf(x - m) > T * D;
}

/*
 * q [B,H,Lq,d] f16; centroids [H,C,d] f16; sizes [H,C].
 * logits [B,H,Lq,C], row_max [B,H,Lq], denom [B,H,Lq], fp32.
 */
void oracle_centroid_score(int B, int H, int Lq, int C, int d, float sm_scale,
                           const uint16_t *q, const uint16_t *centroids, const int32_t *sizes,
                           float *logits, float *row_max, float *denom)
{
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int t = 0; t < Lq; ++t) {
                size_t r = ((size_t)b * H + h) * Lq + t;
                score_one(q + r * d, centroids + (size_t)h * C * d, sizes + (size_t)h * C,
                          NULL, C, d, sm_scale, logits + r * C, row_max + r, denom + r);
            }
}

/*
 * Threshold rule + key ranges.
 * keep_mask [B,H,Lq,ceil(C/32)] (bit i%32 of word i/32), ranges [B,H,Lq,C,2] = (first key,
 * key count) per kept cluster in ascending cluster order, n_ranges, n_keys [B,H,Lq].
 */
void oracle_select(int B, int H, int Lq, int C,
                   const float *logits, const float *row_max, const float *denom,
                   const float *thresh, const int32_t *sizes, const int32_t *offsets,
                   uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys)
{
    int W = (C + 31) / 32;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int t = 0; t < Lq; ++t) {
                size_t r = ((size_t)b * H + h) * Lq + t;
                const float *x = logits + r * C;
                const int32_t *N = sizes + (size_t)h * C;
                const int32_t *off = offsets + (size_t)h * (C + 1);
                uint32_t *mask = keep_mask + r * W;
                int32_t *rg = ranges + r * (size_t)C * 2;
                memset(mask, 0, sizeof(uint32_t) * W);
                int nr = 0, nk = 0;
                for (int i = 0; i < C; ++i) {
                    if (keep_rule(x[i], row_max[r], denom[r], thresh[h], N[i])) {
                        mask[i >> 5] |= 1u << (i & 31);
                        rg[2 * nr] = off[i];
                        rg[2 * nr + 1] = N[i];
                        ++nr;
                        nk += N[i];
                    }
                }
                n_ranges[r] = nr;
                n_keys[r] = nk;
            }
}

/*
 * Prefill selection with averaged scores (Appendix D, "Prefill Stage"): for every (b,h),
 *   Sbar_i = (1/Lq) * sum_t S_i(t),   S_i(t) = exp(x_i(t) - m(t)) / D(t)   (Eq. 1 per query token, fp32),
 * and cluster i is kept iff N_i > 0 and Sbar_i > T (strict).  The average is accumulated in fp64 over t in
 * ascending order.  keep_mask [B,H,ceil(C/32)], ranges [B,H,C,2], n_ranges, n_keys [B,H];
 * mean_scores (may be NULL) [B,H,C] receives Sbar.
 */
void oracle_select_mean(int B, int H, int Lq, int C,
                        const float *logits, const float *row_max, const float *denom,
                        const float *thresh, const int32_t *sizes, const int32_t *offsets,
                        uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                        double *mean_scores)
{
    int W = (C + 31) / 32;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            size_t bh = (size_t)b * H + h;
            const int32_t *N = sizes + (size_t)h * C;
            const int32_t *off = offsets + (size_t)h * (C + 1);
            uint32_t *mask = keep_mask + bh * W;
            int32_t *rg = ranges + bh * (size_t)C * 2;
            memset(mask, 0, sizeof(uint32_t) * W);
            int nr = 0, nk = 0;
            for (int i = 0; i < C; ++i) {
                double acc = 0.0;
                if (N[i] > 0)
                    for (int t = 0; t < Lq; ++t) {
                        size_t r = bh * Lq + t;
                        float S = expf(logits[r * C + i] - row_max[r]) / denom[r];
                        acc += (double)S;
                    }
                double Sbar = acc / (double)Lq;
                if (mean_scores)
                    mean_scores[bh * C + i] = Sbar;
                if (N[i] > 0 && Sbar > (double)thresh[h]) {
                    mask[i >> 5] |= 1u << (i & 31);
                    rg[2 * nr] = off[i];
                    rg[2 * nr + 1] = N[i];
                    ++nr;
                    nk += N[i];
                }
            }
            n_ranges[bh] = nr;
            n_keys[bh] = nk;
        }
}

/*
 * Two-level lookup for one query per (b,h)  (Lq == 1).
 *   level 1: Eq. 2 on (centroids1, sizes1), keep S1 > T1.
 *   candidates: fine clusters child_offsets[j] .. child_offsets[j+1]-1 of every kept j.
 *   level 2: Eq. 3 on the candidates only (max and D over candidates), keep S2 > T2.
 * keep_mask1 [B,H,ceil(C1/32)], keep_mask2 [B,H,ceil(C2/32)], ranges [B,H,C2,2], counts [B,H].
 * logits2 (may be NULL) [B,H,C2]: x of each candidate at its fine-cluster id, NaN elsewhere;
 * stats (may be NULL) [B,H,4] = (m1, D1, m2, D2).
 */
void oracle_hier_select(int B, int H, int C1, int C2, int d, float sm_scale,
                        const uint16_t *q,
                        const uint16_t *centroids1, const int32_t *sizes1, const int32_t *child_offsets,
                        const float *thresh1,
                        const uint16_t *centroids2, const int32_t *sizes2, const int32_t *offsets2,
                        const float *thresh2,
                        uint32_t *keep_mask1, uint32_t *keep_mask2,
                        int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                        float *logits2, float *stats)
{
    int W1 = (C1 + 31) / 32, W2 = (C2 + 31) / 32;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            size_t r = (size_t)b * H + h;
            const uint16_t *qv = q + r * d;
            const int32_t *N1 = sizes1 + (size_t)h * C1;
            const int32_t *co = child_offsets + (size_t)h * (C1 + 1);
            const int32_t *N2 = sizes2 + (size_t)h * C2;
            const int32_t *off2 = offsets2 + (size_t)h * (C2 + 1);
            float *x1 = (float *)malloc(sizeof(float) * (size_t)C1);
            float *x2 = (float *)malloc(sizeof(float) * (size_t)C2);
            int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)C2);
            uint32_t *m1 = keep_mask1 + r * W1, *m2 = keep_mask2 + r * W2;
            memset(m1, 0, sizeof(uint32_t) * W1);
            memset(m2, 0, sizeof(uint32_t) * W2);
            float mx1, D1, mx2 = -INFINITY, D2 = 0.0f;
            score_one(qv, centroids1 + (size_t)h * C1 * d, N1, NULL, C1, d, sm_scale, x1, &mx1, &D1);
            int nc = 0;
            for (int j = 0; j < C1; ++j)
                if (keep_rule(x1[j], mx1, D1, thresh1[h], N1[j])) {
                    m1[j >> 5] |= 1u << (j & 31);
                    for (int l = co[j]; l < co[j + 1]; ++l)
                        cand[nc++] = l;
                }
            if (logits2)
                for (int l = 0; l < C2; ++l)
                    logits2[r * C2 + l] = NAN;
            int nr = 0, nk = 0;
            int32_t *rg = ranges + r * (size_t)C2 * 2;
            if (nc > 0) {
                score_one(qv, centroids2 + (size_t)h * C2 * d, N2, cand, nc, d, sm_scale, x2, &mx2, &D2);
                for (int i = 0; i < nc; ++i) {
                    int l = cand[i];
                    if (logits2)
                        logits2[r * C2 + l] = x2[i];
                    if (keep_rule(x2[i], mx2, D2, thresh2[h], N2[l])) {
                        m2[l >> 5] |= 1u << (l & 31);
                        rg[2 * nr] = off2[l];
                        rg[2 * nr + 1] = N2[l];
                        ++nr;
                        nk += N2[l];
                    }
                }
            }
            n_ranges[r] = nr;
            n_keys[r] = nk;
            if (stats) {
                stats[r * 4 + 0] = mx1;
                stats[r * 4 + 1] = D1;
                stats[r * 4 + 2] = mx2;
                stats[r * 4 + 3] = D2;
            }
            free(x1);
            free(x2);
            free(cand);
        }
}

/*
 * Lookup through a hierarchy of n_levels >= 1 levels of centroids, coarsest first (Section 3.3: Eq. 2 and
 * Eq. 3 applied level after level; the section notes that the two-level scheme extends to more levels).
 *   level 0: scores on all C[0] clusters, keep S > T[0];
 *   level k > 0: candidates = children of the clusters kept at level k-1 (child_offsets[k-1][j] ..
 *   child_offsets[k-1][j+1]-1 for kept j, ascending); scores with the maximum and the normaliser over the
 *   candidates only; keep S > T[k].
 * The last level's child_offsets are key offsets: kept cluster l covers keys [off[l], off[l] + sizes[l]).
 * Per level k: centroids[k] [H, C[k], d] f16, sizes[k] [H, C[k]] (keys under each cluster),
 * child_offsets[k] [H, C[k]+1], thresh[k] [H].  keep_masks[k] (may be NULL) [B, H, ceil(C[k]/32)].
 * ranges [B, H, C[n-1], 2], n_ranges, n_keys [B, H].
 */
void oracle_multilevel_select(int B, int H, int n_levels, const int32_t *C, int d, float sm_scale,
                              const uint16_t *q, const uint16_t *const *centroids, const int32_t *const *sizes,
                              const int32_t *const *child_offsets, const float *const *thresh,
                              uint32_t *const *keep_masks, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys)
{
    int Cmax = 0;
    for (int k = 0; k < n_levels; ++k)
        if (C[k] > Cmax)
            Cmax = C[k];
    const int Cl = C[n_levels - 1];
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h) {
            size_t r = (size_t)b * H + h;
            const uint16_t *qv = q + r * d;
            float *x = (float *)malloc(sizeof(float) * (size_t)Cmax);
            int32_t *cand = (int32_t *)malloc(sizeof(int32_t) * (size_t)Cmax);
            int32_t *next = (int32_t *)malloc(sizeof(int32_t) * (size_t)Cmax);
            int nc = C[0];                       /* level 0: every cluster is a candidate */
            for (int i = 0; i < nc; ++i)
                cand[i] = i;
            int nr = 0, nk = 0;
            int32_t *rg = ranges + r * (size_t)Cl * 2;
            for (int k = 0; k < n_levels; ++k) {
                const int Ck = C[k], Wk = (Ck + 31) / 32;
                const int32_t *Nk = sizes[k] + (size_t)h * Ck;
                const int32_t *co = child_offsets[k] + (size_t)h * (Ck + 1);
                uint32_t *mk = keep_masks && keep_masks[k] ? keep_masks[k] + r * Wk : NULL;
                if (mk)
                    memset(mk, 0, sizeof(uint32_t) * Wk);
                int nn = 0;
                if (nc > 0) {
                    float m, D;
                    score_one(qv, centroids[k] + (size_t)h * Ck * d, Nk, cand, nc, d, sm_scale, x, &m, &D);
                    for (int i = 0; i < nc; ++i) {
                        int j = cand[i];
                        if (!keep_rule(x[i], m, D, thresh[k][h], Nk[j]))
                            continue;
                        if (mk)
                            mk[j >> 5] |= 1u << (j & 31);
                        if (k + 1 < n_levels) {
                            for (int l = co[j]; l < co[j + 1]; ++l)
                                next[nn++] = l;
                        } else {
                            rg[2 * nr] = co[j];
                            rg[2 * nr + 1] = Nk[j];
                            ++nr;
                            nk += Nk[j];
                        }
                    }
                }
                int32_t *t = cand;
                cand = next;
                next = t;
                nc = nn;
            }
            n_ranges[r] = nr;
            n_keys[r] = nk;
            free(x);
            free(cand);
            free(next);
        }
}

static double dot_f64(const uint16_t *a, const uint16_t *b, int d)
{
    double acc = 0.0;
    for (int u = 0; u < d; ++u)
        acc += (double)h2f(a[u]) * (double)h2f(b[u]);
    return acc;
}

/*
 * Exact attention of every query over  (kept fixed keys)  U  (visible user keys), one softmax
 * over the union.  Decode and prefill alike: query t of sequence b sees
 *   fixed keys  j in U_r [start_r, start_r+len_r)  of its own range list, and
 *   user keys   0..U-1            (causal_user == 0)
 *               0..min(t,U-1)     (causal_user != 0: the user input follows the fixed context).
 * K_fixed,V_fixed [H,L,d] shared by all sequences; ranges [B,H,Lq,range_cap,2];
 * K_user,V_user [B,H,U,d].  out [B,H,Lq,d] fp64; lse [B,H,Lq] fp64 = M + log(sum exp(s-M)),
 * -inf (and out = 0) when no key is visible.
 * Only rows r with row_sel == NULL or row_sel[r] != 0 are computed (others left untouched).
 */
void oracle_sparse_attn(int B, int H, int Lq, int L, int U, int d, float sm_scale, int causal_user,
                        int range_cap,
                        const uint16_t *q, const uint16_t *K_fixed, const uint16_t *V_fixed,
                        const int32_t *ranges, const int32_t *n_ranges,
                        const uint16_t *K_user, const uint16_t *V_user,
                        const uint8_t *row_sel, double *out, double *lse)
{
    double scale = (double)sm_scale;
#pragma omp parallel for collapse(3) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b)
        for (int h = 0; h < H; ++h)
            for (int t = 0; t < Lq; ++t) {
                size_t r = ((size_t)b * H + h) * Lq + t;
                if (row_sel && !row_sel[r])
                    continue;
                const uint16_t *qv = q + r * d;
                const uint16_t *Kf = K_fixed + (size_t)h * L * d, *Vf = V_fixed + (size_t)h * L * d;
                const uint16_t *Ku = K_user + ((size_t)b * H + h) * U * d;
                const uint16_t *Vu = V_user + ((size_t)b * H + h) * U * d;
                const int32_t *rg = ranges + r * (size_t)range_cap * 2;
                int nr = n_ranges[r];
                int nu = causal_user ? (t + 1 < U ? t + 1 : U) : U;
                size_t nk = (size_t)nu;
                for (int i = 0; i < nr; ++i)
                    nk += (size_t)rg[2 * i + 1];
                double *o = out + r * d;
                for (int u = 0; u < d; ++u)
                    o[u] = 0.0;
                if (nk == 0) {
                    lse[r] = -INFINITY;
                    continue;
                }
                double *s = (double *)malloc(sizeof(double) * nk);
                size_t n = 0;
                double M = -INFINITY;
                for (int i = 0; i < nr; ++i)
                    for (int j = rg[2 * i]; j < rg[2 * i] + rg[2 * i + 1]; ++j) {
                        s[n] = scale * dot_f64(qv, Kf + (size_t)j * d, d);
                        if (s[n] > M) M = s[n];
                        ++n;
                    }
                for (int j = 0; j < nu; ++j) {
                    s[n] = scale * dot_f64(qv, Ku + (size_t)j * d, d);
                    if (s[n] > M) M = s[n];
                    ++n;
                }
                double sum = 0.0;
                n = 0;
                for (int i = 0; i < nr; ++i)
                    for (int j = rg[2 * i]; j < rg[2 * i] + rg[2 * i + 1]; ++j) {
                        double p = exp(s[n++] - M);
                        sum += p;
                        for (int u = 0; u < d; ++u)
                            o[u] += p * (double)h2f(Vf[(size_t)j * d + u]);
                    }
                for (int j = 0; j < nu; ++j) {
                    double p = exp(s[n++] - M);
                    sum += p;
                    for (int u = 0; u < d; ++u)
                        o[u] += p * (double)h2f(Vu[(size_t)j * d + u]);
                }
                for (int u = 0; u < d; ++u)
                    o[u] /= sum;
                lse[r] = M + log(sum);
                free(s);
            }
}

int oracle_num_threads(void)
{
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp master
        n = omp_get_num_threads();
    }
#endif
    return n;
}
