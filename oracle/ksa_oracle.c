/*
 * ksa_oracle.c -- CPU oracle for Kwai Summary Attention (KSA).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP kernels are checked against.  Nothing in the product path may call it;
 * it shares no code, header, table or helper with the HIP library.
 *
 * What it computes (paper section 2.2 and the distillation section's attention
 * formula): softmax(Q K^T * scale + M_KSA) V over the augmented sequence in
 * which m summary tokens follow every chunk of c text tokens (Eq. 1 with the
 * paper's single summary token generalised to m), where M_KSA lets
 *   - a text token see the text of its own chunk up to itself and of the C
 *     previous chunks, plus the summary tokens of every chunk older than that
 *     window (Eq. 3; summaries of in-window chunks are NOT visible, as the
 *     note under Eq. 3 says);
 *   - a summary token see the text of its own chunk, itself, and the earlier
 *     summary tokens of its own chunk (first bullet of section 2.2.1; the
 *     self and earlier-sibling visibility is this build's reading, flag bit 0
 *     restricts it to self only).
 *
 * Method: every (query, key) pair is tested with the explicit predicate, the
 * whole score row is materialised, softmax is the two-pass max-subtracted
 * definition, all in fp64.  Masked keys receive weight exactly 0.  No tiling,
 * no online softmax, no reordering.
 *
 * Pins: tests/test_oracle_*.py check this file against dense causal attention
 * (single chunk / window covering everything), chunk-aligned sliding windows
 * (Eq. 2), hand-derived masks (tests/golden), closed-form visible counts,
 * softmax invariants, decode == last prefill row, and a pure-Python brute force.
 * The gradients (ksa_oracle_prefill_bwd) are pinned in tests/test_oracle_bwd.py by
 * central differences of this file's own forward pass (every term of the
 * derivative is exercised), by an automatic-differentiation library on the same
 * masked softmax, and by the closed form for a row with a single visible key.
 *
 * Layouts (row-major, contiguous):
 *   prefill  q [B, L, Hq, d]   k, v [B, L, Hkv, d]   float32 (exact bf16 values)
 *            o [B, R, Hq, d]   lse [B, Hq, R]         float64, R = rows requested
 *   backward g [B, L, Hq, d] float32 (upstream gradient); dq like q, dk / dv like k, float64
 *   decode   q [B, Hq, d]; k_sum, v_sum [B, Hkv, S, d]; k_txt, v_txt [B, Hkv, W, d]
 *            text slot t of sequence b holds text index txt_base[b] + t
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define KSA_ORACLE_FLAG_SUMMARY_SELF_ONLY 1u

/* Threads the parallel loops below will use (for reporting next to timings). */
int ksa_oracle_num_threads(void) { return omp_get_max_threads(); }

/* ------------------------------------------------------------------------- */
/* Eq. 1: the augmented sequence.  Position a lies in chunk a / (c+m); the   */
/* first c slots of a chunk are text, the last m are summaries.              */
/* ------------------------------------------------------------------------- */

/*
 * n need not be a whole number of chunks: the paper assumes divisibility to keep its notation short (Sec. 2.2),
 * and a summary exists only once its chunk is complete (cache description, Sec. 2.3.1), so an incomplete last
 * chunk contributes its n mod c text positions and no summaries.  Eq. 1 and Eq. 3 apply to the positions that
 * exist; nothing else changes.
 */
int64_t ksa_oracle_aug_len(int64_t n, int32_t c, int32_t m)
{
    if (c <= 0 || m < 0 || n < 0) return -1;
    return (n / c) * (int64_t)(c + m) + n % c;
}

/*
 * The visibility predicate M_KSA[aq][ak] (1 = visible).
 */
int ksa_oracle_visible(int64_t aq, int64_t ak, int32_t c, int32_t m, int32_t C, uint32_t flags)
{
    const int64_t w = (int64_t)c + m;
    const int64_t jq = aq / w, rq = aq % w;   /* query chunk, slot in chunk */
    const int64_t jk = ak / w, rk = ak % w;   /* key chunk, slot in chunk   */
    const int q_is_summary = rq >= c;
    const int k_is_summary = rk >= c;

    if (!q_is_summary) {
        const int64_t i = jq * c + rq;        /* text index of the query, chunk floor(i/c) = jq */
        if (!k_is_summary) {
            /* Eq. 3 right term: text t_{(floor(i/c)-C)*c} ... t_i, start clamped at 0 */
            const int64_t ik = jk * c + rk;
            int64_t start_chunk = jq - C;
            if (start_chunk < 0) start_chunk = 0;
            return ik >= start_chunk * c && ik <= i;
        }
        /* Eq. 3 left term: summaries s_0 ... s_{floor(i/c)-C-1}, all m slots of those chunks */
        return jk <= jq - (int64_t)C - 1;
    }
    /* summary query: its own chunk only */
    if (jk != jq) return 0;
    if (!k_is_summary) return 1;              /* every text token of the chunk */
    {
        const int64_t uq = rq - c, uk = rk - c;
        if (flags & KSA_ORACLE_FLAG_SUMMARY_SELF_ONLY) return uk == uq;
        return uk <= uq;                      /* itself and earlier summaries of the chunk */
    }
}

void ksa_oracle_mask_row(int64_t aq, int64_t L, int32_t c, int32_t m, int32_t C, uint32_t flags,
                         uint8_t *row_out)
{
    for (int64_t ak = 0; ak < L; ++ak)
        row_out[ak] = (uint8_t)ksa_oracle_visible(aq, ak, c, m, C, flags);
}

/*
 * Index maps of Eq. 1 and the summary position rule (a summary token takes the
 * position id of the last text token of its chunk).  Arrays:
 *   aug_chunk[L], aug_is_summary[L], position_ids[L], text_to_aug[n], summary_to_aug[(n/c)*m]
 */
int ksa_oracle_index_maps(int64_t n, int32_t c, int32_t m, int32_t *aug_chunk, uint8_t *aug_is_summary,
                          int32_t *position_ids, int32_t *text_to_aug, int32_t *summary_to_aug)
{
    const int64_t L = ksa_oracle_aug_len(n, c, m);
    if (L < 0) return -1;
    int64_t a = 0, next_text = 0, next_summary = 0;
    for (int64_t j = 0; j < n / c; ++j) {
        for (int32_t r = 0; r < c; ++r, ++a) {
            aug_chunk[a] = (int32_t)j;
            aug_is_summary[a] = 0;
            position_ids[a] = (int32_t)next_text;
            text_to_aug[next_text++] = (int32_t)a;
        }
        for (int32_t u = 0; u < m; ++u, ++a) {
            aug_chunk[a] = (int32_t)j;
            aug_is_summary[a] = 1;
            position_ids[a] = (int32_t)(next_text - 1);
            summary_to_aug[next_summary++] = (int32_t)a;
        }
    }
    for (int64_t r = 0; r < n % c; ++r, ++a) {   /* the incomplete last chunk: text only */
        aug_chunk[a] = (int32_t)(n / c);
        aug_is_summary[a] = 0;
        position_ids[a] = (int32_t)next_text;
        text_to_aug[next_text++] = (int32_t)a;
    }
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Attention: one row at a time, exactly as the formula is written.          */
/* ------------------------------------------------------------------------- */

static double dot_f32_as_f64(const float *x, const float *y, int32_t d)
{
    double s = 0.0;
    for (int32_t t = 0; t < d; ++t) s += (double)x[t] * (double)y[t];
    return s;
}

/*
 * Weights of one query row over all L keys (0 where masked); returns the
 * log-sum-exp of the visible scaled scores.  `score` is scratch of length L.
 */
static double row_softmax(const float *q_row, const float *k_base, int64_t k_row_stride, int64_t L,
                          int32_t d, double scale, int64_t aq, int32_t c, int32_t m, int32_t C,
                          uint32_t flags, double *score, double *weight)
{
    double mx = -INFINITY;
    for (int64_t ak = 0; ak < L; ++ak) {
        if (ksa_oracle_visible(aq, ak, c, m, C, flags)) {
            score[ak] = scale * dot_f32_as_f64(q_row, k_base + ak * k_row_stride, d);
            if (score[ak] > mx) mx = score[ak];
        }
    }
    double denom = 0.0;
    for (int64_t ak = 0; ak < L; ++ak) {
        if (ksa_oracle_visible(aq, ak, c, m, C, flags)) {
            weight[ak] = exp(score[ak] - mx);
            denom += weight[ak];
        } else {
            weight[ak] = 0.0;
        }
    }
    for (int64_t ak = 0; ak < L; ++ak) weight[ak] /= denom;
    return mx + log(denom);
}

/*
 * Prefill.  rows == NULL computes all L rows (n_rows is then ignored and R = L);
 * otherwise only the listed augmented rows (R = n_rows).  scale <= 0 selects 1/sqrt(d).
 * Returns 0, or -1 on bad arguments.
 */
int ksa_oracle_prefill(const float *q, const float *k, const float *v, int32_t B, int64_t n, int32_t c,
                       int32_t m, int32_t C, int32_t Hq, int32_t Hkv, int32_t d, double scale,
                       uint32_t flags, const int64_t *rows, int64_t n_rows, double *o, double *lse)
{
    const int64_t L = ksa_oracle_aug_len(n, c, m);
    if (L < 0 || B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || C < 0 || Hq % Hkv != 0) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    const int64_t R = rows ? n_rows : L;
    const int32_t group = Hq / Hkv;
    int bad = 0;
    for (int64_t x = 0; rows && x < n_rows; ++x)
        if (rows[x] < 0 || rows[x] >= L) bad = 1;
    if (bad) return -1;

    const int64_t total = (int64_t)B * Hq * R;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
        double *weight = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
#pragma omp for schedule(dynamic, 4)
        for (int64_t item = 0; item < total; ++item) {
            const int64_t x = item % R;
            const int32_t h = (int32_t)((item / R) % Hq);
            const int32_t b = (int32_t)(item / (R * Hq));
            const int64_t aq = rows ? rows[x] : x;
            const int32_t hk = h / group;                 /* GQA: query head h reads KV head h / (Hq/Hkv) */
            const float *q_row = q + (((int64_t)b * L + aq) * Hq + h) * d;
            const float *k_base = k + ((int64_t)b * L * Hkv + hk) * d;
            const float *v_base = v + ((int64_t)b * L * Hkv + hk) * d;
            const int64_t kv_stride = (int64_t)Hkv * d;
            const double l = row_softmax(q_row, k_base, kv_stride, L, d, scale, aq, c, m, C, flags,
                                         score, weight);
            double *o_row = o + (((int64_t)b * R + x) * Hq + h) * d;
            for (int32_t t = 0; t < d; ++t) o_row[t] = 0.0;
            for (int64_t ak = 0; ak < L; ++ak) {
                if (weight[ak] == 0.0) continue;
                const float *v_row = v_base + ak * kv_stride;
                for (int32_t t = 0; t < d; ++t) o_row[t] += weight[ak] * (double)v_row[t];
            }
            if (lse) lse[((int64_t)b * Hq + h) * R + x] = l;
        }
        free(score);
        free(weight);
    }
    return 0;
}

/* Attention weights of one (b, h, aq) row over all L keys, for invariant tests. */
int ksa_oracle_row_weights(const float *q, const float *k, int32_t B, int64_t n, int32_t c, int32_t m,
                           int32_t C, int32_t Hq, int32_t Hkv, int32_t d, double scale, uint32_t flags,
                           int32_t b, int32_t h, int64_t aq, double *weight_out, double *lse_out)
{
    const int64_t L = ksa_oracle_aug_len(n, c, m);
    if (L < 0 || b < 0 || b >= B || h < 0 || h >= Hq || aq < 0 || aq >= L || Hq % Hkv != 0) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    const int32_t hk = h / (Hq / Hkv);
    double *score = (double *)malloc(sizeof(double) * (size_t)L);
    const double l = row_softmax(q + (((int64_t)b * L + aq) * Hq + h) * d,
                                 k + ((int64_t)b * L * Hkv + hk) * d, (int64_t)Hkv * d, L, d, scale, aq,
                                 c, m, C, flags, score, weight_out);
    free(score);
    if (lse_out) *lse_out = l;
    return 0;
}

/* ------------------------------------------------------------------------- */
/* Gradients of the prefill attention (the paper's block-sparse kernel is    */
/* its training kernel as well: section 2.3, Kernel Design; Conclusion).     */
/* The paper prints no backward formula; this is the derivative of the       */
/* definition above, written out.  For an upstream gradient G = dLoss/dO:    */
/*   p_ij   = softmax weight of key j for query i (0 where masked)           */
/*   dV_j   = sum_i p_ij G_i                                                 */
/*   g_ij   = G_i . v_j                       (dLoss/dp_ij)                  */
/*   ds_ij  = p_ij (g_ij - sum_l p_il g_il)   (softmax Jacobian, row i)      */
/*   dQ_i   = scale sum_j ds_ij k_j                                          */
/*   dK_j   = scale sum_i ds_ij q_i                                          */
/* With grouped heads a KV head adds up the contributions of its query heads.*/
/* ------------------------------------------------------------------------- */

/*
 * q_rows == NULL: dq holds all L rows ([B, L, Hq, d]); else the listed augmented rows ([B, n_q_rows, Hq, d]).
 * k_rows == NULL: dk, dv hold all L rows ([B, L, Hkv, d]); else the listed rows ([B, n_k_rows, Hkv, d]).
 * A list of length 0 (non-NULL pointer) skips that output.  g is [B, L, Hq, d] like q.
 * Returns 0, -1 on bad arguments, -3 if memory runs out.
 */
int ksa_oracle_prefill_bwd(const float *q, const float *k, const float *v, const float *g, int32_t B,
                           int64_t n, int32_t c, int32_t m, int32_t C, int32_t Hq, int32_t Hkv, int32_t d,
                           double scale, uint32_t flags, const int64_t *q_rows, int64_t n_q_rows,
                           const int64_t *k_rows, int64_t n_k_rows, double *dq, double *dk, double *dv)
{
    const int64_t L = ksa_oracle_aug_len(n, c, m);
    if (L < 0 || B <= 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || C < 0 || Hq % Hkv != 0) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    const int64_t RQ = q_rows ? n_q_rows : L, RK = k_rows ? n_k_rows : L;
    for (int64_t x = 0; q_rows && x < n_q_rows; ++x)
        if (q_rows[x] < 0 || q_rows[x] >= L) return -1;
    for (int64_t x = 0; k_rows && x < n_k_rows; ++x)
        if (k_rows[x] < 0 || k_rows[x] >= L) return -1;
    const int32_t group = Hq / Hkv;
    const int64_t kv_stride = (int64_t)Hkv * d;

    /* where in the outputs an augmented row goes (-1: not asked for) */
    int64_t *q_slot = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L > 0 ? L : 1));
    int64_t *k_slot = (int64_t *)malloc(sizeof(int64_t) * (size_t)(L > 0 ? L : 1));
    if (!q_slot || !k_slot) { free(q_slot); free(k_slot); return -3; }
    for (int64_t a = 0; a < L; ++a) q_slot[a] = q_rows ? -1 : a, k_slot[a] = k_rows ? -1 : a;
    for (int64_t x = 0; q_rows && x < n_q_rows; ++x) q_slot[q_rows[x]] = x;
    for (int64_t x = 0; k_rows && x < n_k_rows; ++x) k_slot[k_rows[x]] = x;

    for (int64_t x = 0; x < (int64_t)B * RQ * Hq * d; ++x) dq[x] = 0.0;
    for (int64_t x = 0; x < (int64_t)B * RK * Hkv * d; ++x) dk[x] = 0.0, dv[x] = 0.0;

    int failed = 0;
    for (int32_t b = 0; b < B && !failed; ++b)
        for (int32_t h = 0; h < Hq && !failed; ++h) {
            const int32_t hk = h / group;
            const float *k_base = k + ((int64_t)b * L * Hkv + hk) * d;
            const float *v_base = v + ((int64_t)b * L * Hkv + hk) * d;
#pragma omp parallel
            {
                double *score = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
                double *weight = (double *)malloc(sizeof(double) * (size_t)(L > 0 ? L : 1));
                /* this thread's share of dK, dV of head hk; added to the outputs one thread after the other */
                double *pk = (double *)calloc((size_t)(RK > 0 ? RK : 1) * (size_t)d, sizeof(double));
                double *pv = (double *)calloc((size_t)(RK > 0 ? RK : 1) * (size_t)d, sizeof(double));
                if (!score || !weight || !pk || !pv) {
#pragma omp atomic write
                    failed = 1;
                }
#pragma omp barrier
                if (!failed) {
#pragma omp for schedule(dynamic, 4)
                    for (int64_t aq = 0; aq < L; ++aq) {
                        /* does anything asked for depend on this query row? */
                        int wanted = q_slot[aq] >= 0 || !k_rows;
                        for (int64_t x = 0; x < RK && !wanted; ++x)
                            wanted = ksa_oracle_visible(aq, k_rows[x], c, m, C, flags);
                        if (!wanted) continue;
                        const float *q_row = q + (((int64_t)b * L + aq) * Hq + h) * d;
                        const float *g_row = g + (((int64_t)b * L + aq) * Hq + h) * d;
                        row_softmax(q_row, k_base, kv_stride, L, d, scale, aq, c, m, C, flags, score, weight);
                        /* score[] is reused for g_ij */
                        double inner = 0.0;
                        for (int64_t ak = 0; ak < L; ++ak) {
                            if (!ksa_oracle_visible(aq, ak, c, m, C, flags)) continue;
                            score[ak] = dot_f32_as_f64(g_row, v_base + ak * kv_stride, d);
                            inner += weight[ak] * score[ak];
                        }
                        double *dq_row = q_slot[aq] >= 0 ? dq + (((int64_t)b * RQ + q_slot[aq]) * Hq + h) * d : NULL;
                        for (int64_t ak = 0; ak < L; ++ak) {
                            if (!ksa_oracle_visible(aq, ak, c, m, C, flags)) continue;
                            const double ds = weight[ak] * (score[ak] - inner);
                            const float *k_row = k_base + ak * kv_stride;
                            if (dq_row)
                                for (int32_t t = 0; t < d; ++t) dq_row[t] += scale * ds * (double)k_row[t];
                            if (k_slot[ak] >= 0) {
                                double *a_k = pk + k_slot[ak] * d, *a_v = pv + k_slot[ak] * d;
                                for (int32_t t = 0; t < d; ++t) {
                                    a_k[t] += scale * ds * (double)q_row[t];
                                    a_v[t] += weight[ak] * (double)g_row[t];
                                }
                            }
                        }
                    }
#pragma omp critical
                    for (int64_t x = 0; x < RK; ++x) {
                        double *o_k = dk + (((int64_t)b * RK + x) * Hkv + hk) * d;
                        double *o_v = dv + (((int64_t)b * RK + x) * Hkv + hk) * d;
                        for (int32_t t = 0; t < d; ++t) o_k[t] += pk[x * d + t], o_v[t] += pv[x * d + t];
                    }
                }
                free(score);
                free(weight);
                free(pk);
                free(pv);
            }
        }
    free(q_slot);
    free(k_slot);
    return failed ? -3 : 0;
}

/* ------------------------------------------------------------------------- */
/* Decode (section 2.3.1): one new text token per sequence at text index     */
/* pos[b].  Its visible set is Eq. 3 for i = pos: summaries of chunks        */
/* 0 .. floor(i/c)-C-1 and text t_{(floor(i/c)-C)*c} .. t_i.  The set is     */
/* described logically (summary ordinal, text index); the physical order of  */
/* a cache plays no role.                                                    */
/* ------------------------------------------------------------------------- */

static int decode_summary_visible(int64_t i, int64_t u, int32_t c, int32_t m, int32_t C)
{
    /* summary ordinal u is slot u % m of chunk u / m */
    return (u / m) <= i / c - (int64_t)C - 1;
}

static int decode_text_visible(int64_t i, int64_t ik, int32_t c, int32_t C)
{
    int64_t start_chunk = i / c - C;
    if (start_chunk < 0) start_chunk = 0;
    return ik >= start_chunk * c && ik <= i;
}

/*
 * S summary rows (ordinals 0..S-1) and W text rows (text indices txt_base[b] .. txt_base[b]+W-1)
 * are supplied per (b, kv head).  Every visible row must be among them: returns -2 if the
 * supplied rows do not cover the visible set of some sequence, -1 on bad arguments.
 */
int ksa_oracle_decode(const float *q, const float *k_sum, const float *v_sum, int64_t S,
                      const float *k_txt, const float *v_txt, int64_t W, const int64_t *txt_base,
                      const int64_t *pos, int32_t B, int32_t c, int32_t m, int32_t C, int32_t Hq,
                      int32_t Hkv, int32_t d, double scale, double *o, double *lse)
{
    if (B <= 0 || c <= 0 || m < 0 || C < 0 || Hq <= 0 || Hkv <= 0 || d <= 0 || Hq % Hkv != 0) return -1;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)d);
    for (int32_t b = 0; b < B; ++b) {
        const int64_t i = pos[b];
        if (i < 0) return -1;
        int64_t start_chunk = i / c - C;
        if (start_chunk < 0) start_chunk = 0;
        if (txt_base[b] > start_chunk * c || txt_base[b] + W <= i) return -2;
        if (m > 0 && (i / c - C) * (int64_t)m > S) return -2;
    }
    const int32_t group = Hq / Hkv;
    const int64_t total = (int64_t)B * Hq;
    const int64_t N = S + W;
#pragma omp parallel
    {
        double *score = (double *)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
        uint8_t *vis = (uint8_t *)malloc((size_t)(N > 0 ? N : 1));
#pragma omp for schedule(dynamic, 1)
        for (int64_t item = 0; item < total; ++item) {
            const int32_t h = (int32_t)(item % Hq);
            const int32_t b = (int32_t)(item / Hq);
            const int32_t hk = h / group;
            const int64_t i = pos[b];
            const float *q_row = q + ((int64_t)b * Hq + h) * d;
            const float *ks = k_sum + ((int64_t)b * Hkv + hk) * S * d;
            const float *vs = v_sum + ((int64_t)b * Hkv + hk) * S * d;
            const float *kt = k_txt + ((int64_t)b * Hkv + hk) * W * d;
            const float *vt = v_txt + ((int64_t)b * Hkv + hk) * W * d;
            double mx = -INFINITY;
            for (int64_t x = 0; x < N; ++x) {
                const float *k_row;
                if (x < S) {
                    vis[x] = (uint8_t)(m > 0 && decode_summary_visible(i, x, c, m, C));
                    k_row = ks + x * d;
                } else {
                    vis[x] = (uint8_t)decode_text_visible(i, txt_base[b] + (x - S), c, C);
                    k_row = kt + (x - S) * d;
                }
                if (vis[x]) {
                    score[x] = scale * dot_f32_as_f64(q_row, k_row, d);
                    if (score[x] > mx) mx = score[x];
                }
            }
            double denom = 0.0;
            for (int64_t x = 0; x < N; ++x)
                if (vis[x]) denom += exp(score[x] - mx);
            double *o_row = o + ((int64_t)b * Hq + h) * d;
            for (int32_t t = 0; t < d; ++t) o_row[t] = 0.0;
            for (int64_t x = 0; x < N; ++x) {
                if (!vis[x]) continue;
                const double wgt = exp(score[x] - mx) / denom;
                const float *v_row = x < S ? vs + x * d : vt + (x - S) * d;
                for (int32_t t = 0; t < d; ++t) o_row[t] += wgt * (double)v_row[t];
            }
            if (lse) lse[(int64_t)b * Hq + h] = mx + log(denom);
        }
        free(score);
        free(vis);
    }
    return 0;
}
