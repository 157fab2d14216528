/*
 * sv_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, double-precision CPU statement of what one sparse decode
 * step of SparseVILA's decode stage computes (paper section 3.2, "Decode
 * Phase: Query-Aware Retrieval"):
 *
 *   1. score   every cached visual key against the current query,
 *              aggregated over the query heads of one GQA group
 *              (section 3.2, paragraph "Query-Aware Token Selection":
 *              aggregate attention strength between the query and the
 *              visual entries of the KV cache);
 *   2. select  the k visual tokens with the highest relevance score
 *              (same paragraph: the highest-scoring tokens are retained,
 *              the others stay cached but inactive);
 *   3. attend  over all text tokens plus the selected visual tokens
 *              (section 3.2, first paragraph: only the most query-relevant
 *              visual tokens are activated during decoding attention).
 *
 * Only tests, the smoke check and the cpu_baseline leg of the benchmark may
 * call this file.  It shares no code, header, table or helper with the HIP
 * library.  Everything is the written-out definition: no blocking, no
 * split-K, no pre-summed query, no online softmax.
 *
 * Readings where the paper gives no formula (all stated again in the design
 * notes of the repository):
 *   - the aggregate is the SUM over the group's query heads of the scaled
 *     logits scale*<q_h, K_j>; heads are summed AFTER each head's dot product;
 *   - one index set per (batch, kv head); query head h uses kv head h / G;
 *   - k_b = min(k, vis_len[b]); equal scores: the lower index wins; the set is
 *     emitted in ascending index order;
 *   - text tokens are never scored and always attended; one joint softmax over
 *     text followed by the selected visual tokens; no mask, no RoPE.
 *
 * Layout of every tensor: contiguous, row-major, [B, Hkv, N, D] for K and V,
 * [B, Hq, D] for q and out.  dtype 0 = IEEE binary16 bits, 1 = binary32.
 * All inputs are widened EXACTLY to double before any arithmetic.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_pins.py
 * (dense special case against a library attention routine, closed forms,
 * invariants, brute force); nothing is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define SVO_F16 0
#define SVO_F32 1

/* Exact widening of an IEEE-754 binary16 bit pattern. */
double svo_half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double v;
    if (e == 0) {
        v = ldexp((double)f, -24);              /* subnormal: f * 2^-24 */
    } else if (e == 31) {
        v = f ? NAN : INFINITY;
    } else {
        v = ldexp((double)(f | 0x400), e - 25); /* (1024+f) * 2^(e-15-10) */
    }
    return sign ? -v : v;
}

static double load_elem(const void *base, int dtype, int64_t i)
{
    if (dtype == SVO_F16)
        return svo_half_to_double(((const uint16_t *)base)[i]);
    return (double)((const float *)base)[i];
}

static int check_dims(int B, int Hq, int Hkv, int D, int dtype)
{
    if (B < 0 || Hq <= 0 || Hkv <= 0 || D <= 0) return -1;
    if (Hq % Hkv != 0) return -1;
    if (dtype != SVO_F16 && dtype != SVO_F32) return -1;
    return 0;
}

/*
 * Step 1.  scores[b,g,j] = sum_{h in group g} ( scale * sum_d q[b,h,d]*K[b,g,j,d] )
 * for j < vis_len[b]; -inf for vis_len[b] <= j < Nv (padding rows are never
 * read).  vis_len may be NULL (= Nv everywhere).
 */
int svo_score_visual(int B, int Hq, int Hkv, int D, int Nv, int dtype, double scale,
                     const void *q, const void *k_vis, const int32_t *vis_len,
                     double *scores)
{
    if (check_dims(B, Hq, Hkv, D, dtype) || Nv < 0) return -1;
    const int G = Hq / Hkv;
    const int64_t units = (int64_t)B * Hkv;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        const int b = (int)(u / Hkv), g = (int)(u % Hkv);
        const int n = vis_len ? vis_len[b] : Nv;
        for (int j = 0; j < Nv; ++j) {
            double *dst = &scores[(u * Nv) + j];
            if (j >= n) { *dst = -INFINITY; continue; }
            const int64_t krow = ((u * Nv) + j) * (int64_t)D;
            double s = 0.0;
            for (int hh = 0; hh < G; ++hh) {
                const int h = g * G + hh;
                const int64_t qrow = ((int64_t)b * Hq + h) * D;
                double dot = 0.0;
                for (int d = 0; d < D; ++d)
                    dot += load_elem(q, dtype, qrow + d) * load_elem(k_vis, dtype, krow + d);
                s += scale * dot;
            }
            *dst = s;
        }
    }
    return 0;
}

/* ---- Step 2: full sort by (score descending, index ascending). ---- */
typedef struct { double s; int32_t j; } svo_pair;

static int cmp_score_desc_index_asc(const void *a, const void *b)
{
    const svo_pair *x = (const svo_pair *)a, *y = (const svo_pair *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int cmp_int32_asc(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/*
 * idx[b,g,0..count) = the k_b = min(k, vis_len[b]) indices of the largest
 * scores among j < vis_len[b], ties to the lower index, ascending; slots
 * count..k-1 hold -1.  count[b,g] = k_b.
 */
int svo_topk_select(int B, int Hkv, int Nv, int k, const double *scores,
                    const int32_t *vis_len, int32_t *idx, int32_t *count)
{
    if (B < 0 || Hkv <= 0 || Nv < 0 || k < 0) return -1;
    const int64_t units = (int64_t)B * Hkv;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t u = 0; u < units; ++u) {
        const int b = (int)(u / Hkv);
        const int n = vis_len ? vis_len[b] : Nv;
        const int kb = k < n ? k : n;
        svo_pair *p = (svo_pair *)malloc(sizeof(svo_pair) * (size_t)(n > 0 ? n : 1));
        if (!p) { fail = 1; continue; }
        for (int j = 0; j < n; ++j) { p[j].s = scores[u * Nv + j]; p[j].j = j; }
        qsort(p, (size_t)n, sizeof(svo_pair), cmp_score_desc_index_asc);
        int32_t *o = &idx[u * k];
        for (int i = 0; i < kb; ++i) o[i] = p[i].j;
        qsort(o, (size_t)kb, sizeof(int32_t), cmp_int32_asc);
        for (int i = kb; i < k; ++i) o[i] = -1;
        count[u] = kb;
        free(p);
    }
    return fail ? -2 : 0;
}

/*
 * Step 3.  For every query head h (kv head g = h / G): the token list T is the
 * text tokens i < txt_len[b] followed by the visual tokens idx[b,g,0..count);
 * l_t = scale*<q_h, key_t>, m = max l_t, w_t = exp(l_t - m), Z = sum w_t,
 * out[b,h,:] = sum_t w_t*value_t / Z, lse[b,h] = m + log Z.
 * wsum[b,h] (optional) = sum_t (w_t / Z): the total softmax mass, for the
 * "weights sum to one" pin.  Empty T gives out = 0, lse = -inf, wsum = 0.
 */
int svo_sparse_decode_attn(int B, int Hq, int Hkv, int D, int Nv, int Nt, int k,
                           int dtype, double scale, const void *q,
                           const void *k_vis, const void *v_vis,
                           const void *k_txt, const void *v_txt,
                           const int32_t *txt_len,
                           const int32_t *idx, const int32_t *count,
                           double *out, double *lse, double *wsum)
{
    if (check_dims(B, Hq, Hkv, D, dtype) || Nv < 0 || Nt < 0 || k < 0) return -1;
    const int G = Hq / Hkv;
    const int64_t heads = (int64_t)B * Hq;
    int fail = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < heads; ++bh) {
        const int b = (int)(bh / Hq), h = (int)(bh % Hq), g = h / G;
        const int64_t u = (int64_t)b * Hkv + g;
        const int nt = txt_len ? txt_len[b] : Nt;
        const int kc = (k > 0 && count) ? count[u] : 0;
        const int T = nt + kc;
        double *o = &out[bh * D];
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (T == 0) {
            if (lse) lse[bh] = -INFINITY;
            if (wsum) wsum[bh] = 0.0;
            continue;
        }
        double *logit = (double *)malloc(sizeof(double) * (size_t)T);
        int64_t *krow = (int64_t *)malloc(sizeof(int64_t) * (size_t)T);
        if (!logit || !krow) { fail = 1; free(logit); free(krow); continue; }
        /* row offsets (in elements) of each token of T; text rows are tagged
         * with a negative offset so the two caches stay apart */
        for (int t = 0; t < T; ++t) {
            if (t < nt) krow[t] = -(((u * Nt) + t) * (int64_t)D) - 1;
            else        krow[t] = ((u * Nv) + idx[u * k + (t - nt)]) * (int64_t)D;
        }
        const int64_t qrow = bh * D;
        double m = -INFINITY;
        for (int t = 0; t < T; ++t) {
            const int is_txt = krow[t] < 0;
            const int64_t r = is_txt ? -(krow[t] + 1) : krow[t];
            const void *kb = is_txt ? k_txt : k_vis;
            double dot = 0.0;
            for (int d = 0; d < D; ++d)
                dot += load_elem(q, dtype, qrow + d) * load_elem(kb, dtype, r + d);
            logit[t] = scale * dot;
            if (logit[t] > m) m = logit[t];
        }
        double Z = 0.0;
        for (int t = 0; t < T; ++t) Z += exp(logit[t] - m);
        double mass = 0.0;
        for (int t = 0; t < T; ++t) {
            const int is_txt = krow[t] < 0;
            const int64_t r = is_txt ? -(krow[t] + 1) : krow[t];
            const void *vb = is_txt ? v_txt : v_vis;
            const double w = exp(logit[t] - m) / Z;
            mass += w;
            for (int d = 0; d < D; ++d) o[d] += w * load_elem(vb, dtype, r + d);
        }
        if (lse) lse[bh] = m + log(Z);
        if (wsum) wsum[bh] = mass;
        free(logit);
        free(krow);
    }
    return fail ? -2 : 0;
}

/*
 * The whole step: 1 -> 2 -> 3 on the same inputs.  scores [B,Hkv,Nv] double,
 * idx [B,Hkv,k], count [B,Hkv], out [B,Hq,D] double, lse/wsum [B,Hq] or NULL.
 */
int svo_decode_step(int B, int Hq, int Hkv, int D, int Nv, int Nt, int k,
                    int dtype, double scale, const void *q,
                    const void *k_vis, const void *v_vis,
                    const void *k_txt, const void *v_txt,
                    const int32_t *vis_len, const int32_t *txt_len,
                    double *scores, int32_t *idx, int32_t *count,
                    double *out, double *lse, double *wsum)
{
    int rc = svo_score_visual(B, Hq, Hkv, D, Nv, dtype, scale, q, k_vis, vis_len, scores);
    if (rc) return rc;
    rc = svo_topk_select(B, Hkv, Nv, k, scores, vis_len, idx, count);
    if (rc) return rc;
    return svo_sparse_decode_attn(B, Hq, Hkv, D, Nv, Nt, k, dtype, scale, q,
                                  k_vis, v_vis, k_txt, v_txt, txt_len,
                                  idx, count, out, lse, wsum);
}
