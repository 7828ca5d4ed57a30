/*
 * CPU ORACLE for the DSV two-stage sparse attention path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision statement of what the path computes, written from the
 * paper's definitions.  It shares no code, header, table or helper with the HIP library and
 * must never be linked, imported or called by it; only the tests, the smoke check and the
 * benchmark's cpu_baseline leg use it.
 *
 * What is defined where (paper: "DSV: Exploiting Dynamic Sparsity to Accelerate Large-Scale
 * Video DiT Training"):
 *   - low-rank projection Q_lr = Q Wq, K_lr = K Wk ......... Sec. "Low-Rank based Sparsity Prediction"
 *   - approximate scores Q_lr K_lr^T and per-query top-k .... Sec. "Critical KV Estimation with Kernel Fusion"
 *   - attention over only the selected (critical) KV ........ Sec. "Sparse Attention with Query Grouping",
 *                                                             with softmax(QK^T/sqrt(d_k))V from
 *                                                             Sec. "Various Self-Attention Paradigms"
 *   - dense attention (the k = L limit and the comparator) .. Sec. "Various Self-Attention Paradigms"
 *   - query groups sharing one index row (3D cubes, centre query as proxy): same section as the sparse
 *     attention, defined further down in this file
 *
 * Readings taken where the paper is silent (listed again in the design notes):
 *   - one (Wq, Wk) pair per head, applied to that head's Q and K;
 *   - projected values are rounded (nearest-even) to the storage dtype, scores are exact sums;
 *   - the k largest scores win, equal scores go to the lower key index, rows are emitted in
 *     ascending key index; exactly k indices per query, no mask, no forced keys;
 *   - softmax is normalised over the selected subset only; lse is that subset's log-sum-exp;
 *   - no gradient flows through the selection or the predictor (the predictor is trained
 *     outside the main graph), so backward returns dQ, dK, dV only.
 *
 * Inputs are float arrays that already hold storage-dtype-rounded values; all arithmetic is
 * in double.  Loops follow the formulas literally: no blocking, no fusion.  OpenMP is used
 * only across independent query rows (or keys), never inside a sum.
 *
 * Parity pins (tests/test_oracle_*.py): textbook GEMM for the projection, brute-force
 * lexicographic sort for the selection, dense softmax attention and library autograd at
 * k = L, closed forms (k = 1, Q = 0, all-equal scores), softmax and gradient identities,
 * central finite differences.  No function here is unpinned.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define DSV_ORACLE_F32 0
#define DSV_ORACLE_BF16 1

/* Round a double to a binary format with `prec` significand bits (24: fp32, 8: bf16) and
 * minimum subnormal exponent `emin_sub` (fp32: -149, bf16: -133), nearest-even, straight
 * from the double (no intermediate fp32 rounding). */
static double round_to_format(double x, int prec, int emin_sub)
{
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    (void)frexp(x, &e);            /* |x| = m * 2^e with 0.5 <= m < 1 */
    int ulp_exp = e - prec;        /* weight of the last kept bit */
    if (ulp_exp < emin_sub) ulp_exp = emin_sub;
    double q = nearbyint(ldexp(x, -ulp_exp));   /* default rounding mode: nearest-even */
    return ldexp(q, ulp_exp);
}

double dsv_oracle_round(double x, int dtype)
{
    return dtype == DSV_ORACLE_BF16 ? round_to_format(x, 8, -133) : round_to_format(x, 24, -149);
}

/* Projection of n token rows: out[i, t] = rnd( sum_c X[i, c] * W[c, t] ).
 * X [n, d], W [d, r], out [n, r] (float holding the rounded value). */
void dsv_oracle_project(const float *X, const float *W, int64_t n, int d, int r, int dtype, float *out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        for (int t = 0; t < r; ++t) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += (double)X[i * d + c] * (double)W[(int64_t)c * r + t];
            out[i * r + t] = (float)dsv_oracle_round(acc, dtype);
        }
    }
}

/* Approximate scores of nq query rows against all L keys: S[i, j] = sum_t Qlr[i, t] * Klr[j, t].
 * No scale and no softmax: the ranking is invariant to both. */
void dsv_oracle_scores(const float *Qlr, const float *Klr, int64_t nq, int64_t L, int r, double *S)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < nq; ++i) {
        for (int64_t j = 0; j < L; ++j) {
            double acc = 0.0;
            for (int t = 0; t < r; ++t) acc += (double)Qlr[i * r + t] * (double)Klr[j * r + t];
            S[i * L + j] = acc;
        }
    }
}

typedef struct { double s; int32_t j; } scored_key;

/* Total order of the selection: higher score first, equal scores -> lower index first. */
static int cmp_score_desc_index_asc(const void *a, const void *b)
{
    const scored_key *x = (const scored_key *)a, *y = (const scored_key *)b;
    if (x->s > y->s) return -1;
    if (x->s < y->s) return 1;
    return (x->j > y->j) - (x->j < y->j);
}

static int cmp_int32(const void *a, const void *b)
{
    int32_t x = *(const int32_t *)a, y = *(const int32_t *)b;
    return (x > y) - (x < y);
}

/* Selection on given score rows: idx[i, :] = the k keys first in the total order above,
 * written in ascending key index.  S [nq, L] (any real-valued scores), idx [nq, k].
 * Full sort of every row: the definition, not a streaming algorithm. */
void dsv_oracle_topk_from_scores(const double *S, int64_t nq, int64_t L, int64_t k, int32_t *idx)
{
#pragma omp parallel
    {
        scored_key *row = (scored_key *)malloc((size_t)L * sizeof(scored_key));
#pragma omp for schedule(dynamic, 4)
        for (int64_t i = 0; i < nq; ++i) {
            for (int64_t j = 0; j < L; ++j) { row[j].s = S[i * L + j]; row[j].j = (int32_t)j; }
            qsort(row, (size_t)L, sizeof(scored_key), cmp_score_desc_index_asc);
            for (int64_t t = 0; t < k; ++t) idx[i * k + t] = row[t].j;
            qsort(idx + i * k, (size_t)k, sizeof(int32_t), cmp_int32);
        }
        free(row);
    }
}

/* Stage 1 for nq query rows of one head, end to end: project the given query rows and all L
 * keys, score, select.  Q [nq, d] (the chosen rows), K [L, d], Wq, Wk [d, r].
 * Optional outputs (may be NULL): Qlr_out [nq, r], Klr_out [L, r], S_out [nq, L]. */
void dsv_oracle_lowrank_topk(const float *Q, const float *K, const float *Wq, const float *Wk,
                             int64_t nq, int64_t L, int d, int r, int64_t k, int dtype,
                             int32_t *idx, float *Qlr_out, float *Klr_out, double *S_out)
{
    float *Qlr = Qlr_out ? Qlr_out : (float *)malloc((size_t)nq * r * sizeof(float));
    float *Klr = Klr_out ? Klr_out : (float *)malloc((size_t)L * r * sizeof(float));
    double *S = S_out ? S_out : (double *)malloc((size_t)nq * L * sizeof(double));
    dsv_oracle_project(Q, Wq, nq, d, r, dtype, Qlr);
    dsv_oracle_project(K, Wk, L, d, r, dtype, Klr);
    dsv_oracle_scores(Qlr, Klr, nq, L, r, S);
    dsv_oracle_topk_from_scores(S, nq, L, k, idx);
    if (!Qlr_out) free(Qlr);
    if (!Klr_out) free(Klr);
    if (!S_out) free(S);
}

/* Sparse attention forward for nq query rows.  Q [nq, d] (the chosen rows), K, V [L, d],
 * idx [nq, k] (distinct keys per row, any order).
 *   s_j = scale * q . k_j          for j in idx[i]
 *   lse = log sum_j exp(s_j)       (computed as m + log sum exp(s_j - m), m = max_j s_j)
 *   p_j = exp(s_j - lse),  O_i = sum_j p_j v_j
 * Outputs: O [nq, d], lse [nq]; P [nq, k] optional (NULL to skip), in idx order. */
void dsv_oracle_sparse_fwd(const float *Q, const float *K, const float *V, const int32_t *idx,
                           int64_t nq, int64_t L, int d, int64_t k, double scale,
                           double *O, double *lse, double *P)
{
    (void)L;
#pragma omp parallel
    {
        double *s = (double *)malloc((size_t)k * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < nq; ++i) {
            const int32_t *row = idx + i * k;
            double m = -INFINITY;
            for (int64_t t = 0; t < k; ++t) {
                const float *kj = K + (int64_t)row[t] * d;
                double acc = 0.0;
                for (int c = 0; c < d; ++c) acc += (double)Q[i * d + c] * (double)kj[c];
                s[t] = scale * acc;
                if (s[t] > m) m = s[t];
            }
            double z = 0.0;
            for (int64_t t = 0; t < k; ++t) z += exp(s[t] - m);
            double l = m + log(z);
            lse[i] = l;
            for (int c = 0; c < d; ++c) O[i * d + c] = 0.0;
            for (int64_t t = 0; t < k; ++t) {
                double p = exp(s[t] - l);
                if (P) P[i * k + t] = p;
                const float *vj = V + (int64_t)row[t] * d;
                for (int c = 0; c < d; ++c) O[i * d + c] += p * (double)vj[c];
            }
        }
        free(s);
    }
}

/* Per-pair terms of the backward, shared by the routines below.
 *   Delta = dO_i . O_i ;  dP_j = dO_i . v_j ;  p_j = exp(scale q_i . k_j - lse_i) ;  dS_j = p_j (dP_j - Delta) */
static double row_delta(const float *dOi, const double *Oi, int d)
{
    double delta = 0.0;
    for (int c = 0; c < d; ++c) delta += (double)dOi[c] * Oi[c];
    return delta;
}

static void pair_p_and_ds(const float *q, const float *dOi, double delta, double lse_i, const float *kj,
                          const float *vj, int d, double scale, double *p, double *dS)
{
    double acc = 0.0, dp = 0.0;
    for (int c = 0; c < d; ++c) acc += (double)q[c] * (double)kj[c];
    for (int c = 0; c < d; ++c) dp += (double)dOi[c] * (double)vj[c];
    *p = exp(scale * acc - lse_i);
    *dS = *p * (dp - delta);
}

/* q, dOi, Oi [d]; writes p[t], dS[t] for the k selected keys of this row. */
static void row_p_and_ds(const float *q, const float *dOi, const double *Oi, double lse_i,
                         const float *K, const float *V, const int32_t *row, int d, int64_t k,
                         double scale, double *p, double *dS)
{
    const double delta = row_delta(dOi, Oi, d);
    for (int64_t t = 0; t < k; ++t)
        pair_p_and_ds(q, dOi, delta, lse_i, K + (int64_t)row[t] * d, V + (int64_t)row[t] * d, d, scale, &p[t], &dS[t]);
}

/* Sparse attention backward (selection held constant) for nq query rows of one head: their dQ,
 * and their contributions to dK and dV.  With nq = L and all rows given this is the whole head.
 * Q, dO, O [nq, d], lse [nq], idx [nq, k] are the rows' data (O, lse: the oracle's own forward
 * results in double); K, V [L, d].  Outputs: dQ [nq, d] (overwritten); dK, dV [L, d] are
 * ACCUMULATED INTO (the caller zeroes them), so that keys no query selected stay exactly zero:
 *   dQ_i = scale * sum_j dS_ij k_j
 *   dK_j = scale * sum_{i : j in idx[i]} dS_ij q_i
 *   dV_j =         sum_{i : j in idx[i]} p_ij  dO_i
 * Serial over queries: the scatter into dK, dV is written exactly as the sums above read. */
void dsv_oracle_sparse_bwd_rows(const float *Q, const float *K, const float *V, const int32_t *idx,
                                const double *O, const double *lse, const float *dO,
                                int64_t nq, int d, int64_t k, double scale,
                                double *dQ, double *dK, double *dV)
{
    double *p = (double *)malloc((size_t)k * sizeof(double));
    double *dS = (double *)malloc((size_t)k * sizeof(double));
    memset(dQ, 0, (size_t)nq * d * sizeof(double));
    for (int64_t i = 0; i < nq; ++i) {
        const int32_t *row = idx + i * k;
        row_p_and_ds(Q + i * d, dO + i * d, O + i * d, lse[i], K, V, row, d, k, scale, p, dS);
        for (int64_t t = 0; t < k; ++t) {
            int64_t j = row[t];
            for (int c = 0; c < d; ++c) {
                dQ[i * d + c] += scale * dS[t] * (double)K[j * d + c];
                dK[j * d + c] += scale * dS[t] * (double)Q[i * d + c];
                dV[j * d + c] += p[t] * (double)dO[i * d + c];
            }
        }
    }
    free(p);
    free(dS);
}

/* Whole head: Q, K, V, dO, O [L, d], idx [L, k], lse [L] -> dQ, dK, dV [L, d]. */
void dsv_oracle_sparse_bwd(const float *Q, const float *K, const float *V, const int32_t *idx,
                           const double *O, const double *lse, const float *dO,
                           int64_t L, int d, int64_t k, double scale,
                           double *dQ, double *dK, double *dV)
{
    memset(dK, 0, (size_t)L * d * sizeof(double));
    memset(dV, 0, (size_t)L * d * sizeof(double));
    dsv_oracle_sparse_bwd_rows(Q, K, V, idx, O, lse, dO, L, d, k, scale, dQ, dK, dV);
}

/* dQ for nq chosen query rows only (same formulas).  Q, dO, O [nq, d] and lse [nq] are the
 * chosen rows; K, V [L, d]; idx [nq, k]. */
void dsv_oracle_sparse_bwd_dq_rows(const float *Q, const float *K, const float *V, const int32_t *idx,
                                   const double *O, const double *lse, const float *dO,
                                   int64_t nq, int d, int64_t k, double scale, double *dQ)
{
#pragma omp parallel
    {
        double *p = (double *)malloc((size_t)k * sizeof(double));
        double *dS = (double *)malloc((size_t)k * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t i = 0; i < nq; ++i) {
            const int32_t *row = idx + i * k;
            row_p_and_ds(Q + i * d, dO + i * d, O + i * d, lse[i], K, V, row, d, k, scale, p, dS);
            for (int c = 0; c < d; ++c) dQ[i * d + c] = 0.0;
            for (int64_t t = 0; t < k; ++t)
                for (int c = 0; c < d; ++c)
                    dQ[i * d + c] += scale * dS[t] * (double)K[(int64_t)row[t] * d + c];
        }
        free(p);
        free(dS);
    }
}

/* dK_j and dV_j for ONE key j, given the n queries that selected it.  For each such query the
 * caller passes its row data: Qs, dOs, Os [n, d], lses [n], and its index row idxs [n, k]
 * (every row contains j).  K, V [L, d].  Outputs dKj, dVj [d].
 * Each query's term (scale dS_aj q_a and p_aj dO_a) is formed independently (OpenMP across the
 * queries), then the terms are summed in query order. */
void dsv_oracle_sparse_bwd_dkdv_key(int32_t j, const float *Qs, const float *dOs, const double *Os,
                                    const double *lses, const int32_t *idxs, int64_t n,
                                    const float *K, const float *V, int d, int64_t k, double scale,
                                    double *dKj, double *dVj)
{
    double *termK = (double *)calloc((size_t)n * d, sizeof(double));
    double *termV = (double *)calloc((size_t)n * d, sizeof(double));
    (void)k;
#pragma omp parallel for schedule(static)
    for (int64_t a = 0; a < n; ++a) {
        const int32_t *row = idxs + a * k;
        const double delta = row_delta(dOs + a * d, Os + a * d, d);
        for (int64_t t = 0; t < k; ++t) {
            if (row[t] != j) continue;   /* only the pair (query a, key j) enters dK_j and dV_j */
            double p, dS;
            pair_p_and_ds(Qs + a * d, dOs + a * d, delta, lses[a], K + (int64_t)j * d, V + (int64_t)j * d, d, scale, &p, &dS);
            for (int c = 0; c < d; ++c) {
                termK[a * d + c] += scale * dS * (double)Qs[a * d + c];
                termV[a * d + c] += p * (double)dOs[a * d + c];
            }
        }
    }
    for (int c = 0; c < d; ++c) { dKj[c] = 0.0; dVj[c] = 0.0; }
    for (int64_t a = 0; a < n; ++a)
        for (int c = 0; c < d; ++c) { dKj[c] += termK[a * d + c]; dVj[c] += termV[a * d + c]; }
    free(termK);
    free(termV);
}

/* Dense (full, non-causal) attention of one head, brute force: the L x L probability matrix
 * is materialised.  Q, K, V [L, d] -> O [L, d], lse [L], P [L, L] (optional). */
void dsv_oracle_dense_fwd(const float *Q, const float *K, const float *V, int64_t L, int d,
                          double scale, double *O, double *lse, double *P)
{
    double *s = (double *)malloc((size_t)L * sizeof(double));
    for (int64_t i = 0; i < L; ++i) {
        double m = -INFINITY;
        for (int64_t j = 0; j < L; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += (double)Q[i * d + c] * (double)K[j * d + c];
            s[j] = scale * acc;
            if (s[j] > m) m = s[j];
        }
        double z = 0.0;
        for (int64_t j = 0; j < L; ++j) z += exp(s[j] - m);
        lse[i] = m + log(z);
        for (int c = 0; c < d; ++c) O[i * d + c] = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double p = exp(s[j] - lse[i]);
            if (P) P[i * L + j] = p;
            for (int c = 0; c < d; ++c) O[i * d + c] += p * (double)V[j * d + c];
        }
    }
    free(s);
}

/* Gradient of dense attention, from the materialised P:  dV = P^T dO;  dP = dO V^T;
 * dS = P o (dP - rowsum(dO o O));  dQ = scale dS K;  dK = scale dS^T Q. */
void dsv_oracle_dense_bwd(const float *Q, const float *K, const float *V, const float *dO,
                          int64_t L, int d, double scale, double *dQ, double *dK, double *dV)
{
    double *O = (double *)malloc((size_t)L * d * sizeof(double));
    double *lse = (double *)malloc((size_t)L * sizeof(double));
    double *P = (double *)malloc((size_t)L * L * sizeof(double));
    dsv_oracle_dense_fwd(Q, K, V, L, d, scale, O, lse, P);
    memset(dQ, 0, (size_t)L * d * sizeof(double));
    memset(dK, 0, (size_t)L * d * sizeof(double));
    memset(dV, 0, (size_t)L * d * sizeof(double));
    for (int64_t i = 0; i < L; ++i) {
        double delta = 0.0;
        for (int c = 0; c < d; ++c) delta += (double)dO[i * d + c] * O[i * d + c];
        for (int64_t j = 0; j < L; ++j) {
            double dp = 0.0;
            for (int c = 0; c < d; ++c) dp += (double)dO[i * d + c] * (double)V[j * d + c];
            double p = P[i * L + j];
            double ds = p * (dp - delta);
            for (int c = 0; c < d; ++c) {
                dQ[i * d + c] += scale * ds * (double)K[j * d + c];
                dK[j * d + c] += scale * ds * (double)Q[i * d + c];
                dV[j * d + c] += p * (double)dO[i * d + c];
            }
        }
    }
    free(O);
    free(lse);
    free(P);
}

/* ---------------------------------------------------------------------------------------------
 * Query grouping (Sec. "Sparse Attention with Query Grouping"; Observation 5: neighbouring tokens of
 * the 3D latent grid attend to similar keys).  Tokens lie on a grid of F x Hh x Ww, flattened frames
 * first, then height, then width (Sec. "Various Self-Attention Paradigms", footnote on the token
 * order).  The grid is tiled by cubes of gf x gh x gw voxels; the G = gf*gh*gw queries of a cube form
 * a group, the group's centre query alone is scored against all keys, and its k best keys are the
 * index row shared by every member.  Readings: cubes tile the grid exactly (sizes divide); the
 * "central" voxel of a cube with an even side is the one at offset side/2 (for 2 x 2 x 2: offset
 * (1, 1, 1)); groups are numbered in the same frames-height-width order as tokens, members likewise
 * inside their cube.
 * ------------------------------------------------------------------------------------------- */

/* Token index of member m of group g.  Returns -1 if the cube sizes do not divide the grid. */
int64_t dsv_oracle_group_member(int64_t g, int m, int F, int Hh, int Ww, int gf, int gh, int gw)
{
    if (F % gf || Hh % gh || Ww % gw) return -1;
    const int nh = Hh / gh, nw = Ww / gw;
    const int64_t cf = g / ((int64_t)nh * nw), ch = (g / nw) % nh, cw = g % nw;   /* cube coordinates */
    const int mf = m / (gh * gw), mh = (m / gw) % gh, mw = m % gw;                /* offset in the cube */
    const int64_t f = cf * gf + mf, h = ch * gh + mh, w = cw * gw + mw;
    return (f * Hh + h) * Ww + w;
}

/* Member number of the centre (proxy) query of every cube. */
int dsv_oracle_group_centre(int gf, int gh, int gw)
{
    return ((gf / 2) * gh + gh / 2) * gw + gw / 2;
}

/* Grouped selection for one head: idx_g [n_groups, k] = the k best keys of each group's centre
 * query (same total order and row order as the per-query selection).  Q, K [L, d], L = F*Hh*Ww. */
void dsv_oracle_lowrank_topk_grouped(const float *Q, const float *K, const float *Wq, const float *Wk,
                                     int F, int Hh, int Ww, int gf, int gh, int gw, int d, int r, int64_t k,
                                     int dtype, int32_t *idx_g)
{
    const int64_t L = (int64_t)F * Hh * Ww;
    const int G = gf * gh * gw;
    const int64_t ng = L / G;
    const int centre = dsv_oracle_group_centre(gf, gh, gw);
    float *Qc = (float *)malloc((size_t)ng * d * sizeof(float));
    for (int64_t g = 0; g < ng; ++g) {
        const int64_t i = dsv_oracle_group_member(g, centre, F, Hh, Ww, gf, gh, gw);
        memcpy(Qc + g * d, Q + i * d, (size_t)d * sizeof(float));
    }
    dsv_oracle_lowrank_topk(Qc, K, Wq, Wk, ng, L, d, r, k, dtype, idx_g, NULL, NULL, NULL);
    free(Qc);
}

/* The per-query index that grouping stands for: row i = the row of i's group.  idx [L, k]. */
void dsv_oracle_group_expand_idx(const int32_t *idx_g, int F, int Hh, int Ww, int gf, int gh, int gw, int64_t k,
                                 int32_t *idx)
{
    const int64_t L = (int64_t)F * Hh * Ww;
    const int G = gf * gh * gw;
    for (int64_t g = 0; g < L / G; ++g)
        for (int m = 0; m < G; ++m) {
            const int64_t i = dsv_oracle_group_member(g, m, F, Hh, Ww, gf, gh, gw);
            memcpy(idx + i * k, idx_g + g * k, (size_t)k * sizeof(int32_t));
        }
}

/* Grouped sparse attention of one head: every member of a group attends over the group's shared
 * index row -- by definition the per-query routines on the expanded index. */
void dsv_oracle_sparse_fwd_grouped(const float *Q, const float *K, const float *V, const int32_t *idx_g,
                                   int F, int Hh, int Ww, int gf, int gh, int gw, int d, int64_t k, double scale,
                                   double *O, double *lse)
{
    const int64_t L = (int64_t)F * Hh * Ww;
    int32_t *idx = (int32_t *)malloc((size_t)L * k * sizeof(int32_t));
    dsv_oracle_group_expand_idx(idx_g, F, Hh, Ww, gf, gh, gw, k, idx);
    dsv_oracle_sparse_fwd(Q, K, V, idx, L, L, d, k, scale, O, lse, NULL);
    free(idx);
}

void dsv_oracle_sparse_bwd_grouped(const float *Q, const float *K, const float *V, const int32_t *idx_g,
                                   const float *dO, int F, int Hh, int Ww, int gf, int gh, int gw, int d, int64_t k,
                                   double scale, double *dQ, double *dK, double *dV)
{
    const int64_t L = (int64_t)F * Hh * Ww;
    int32_t *idx = (int32_t *)malloc((size_t)L * k * sizeof(int32_t));
    double *O = (double *)malloc((size_t)L * d * sizeof(double)), *lse = (double *)malloc((size_t)L * sizeof(double));
    dsv_oracle_group_expand_idx(idx_g, F, Hh, Ww, gf, gh, gw, k, idx);
    dsv_oracle_sparse_fwd(Q, K, V, idx, L, L, d, k, scale, O, lse, NULL);
    dsv_oracle_sparse_bwd(Q, K, V, idx, O, lse, dO, L, d, k, scale, dQ, dK, dV);
    free(idx); free(O); free(lse);
}

/* Offline profiling of the group size (Sec. "Sparse Attention with Query Grouping": the largest cube whose queries
 * share a required ratio, e.g. 80 %, of their critical keys): for one head, given the PER-QUERY index idx [L, k]
 * (rows = sets of distinct keys, any order), the number of (query, key) pairs whose key is also in the row of the
 * query's group centre,
 *     count = sum_i | row(i) intersect row(centre of i's group) |,
 * so that count / (L k) is the mean share of a query's own selection that the shared row would keep (a centre query
 * contributes k).  Returns -1 if the cube does not tile the grid. */
int64_t dsv_oracle_group_overlap(const int32_t *idx, int F, int Hh, int Ww, int gf, int gh, int gw, int64_t k)
{
    if (F % gf || Hh % gh || Ww % gw) return -1;
    const int64_t L = (int64_t)F * Hh * Ww;
    const int G = gf * gh * gw;
    const int centre = dsv_oracle_group_centre(gf, gh, gw);
    unsigned char *in_centre = (unsigned char *)calloc((size_t)L, 1);
    int64_t count = 0;
    for (int64_t g = 0; g < L / G; ++g) {
        const int32_t *crow = idx + dsv_oracle_group_member(g, centre, F, Hh, Ww, gf, gh, gw) * k;
        for (int64_t t = 0; t < k; ++t) in_centre[crow[t]] = 1;
        for (int m = 0; m < G; ++m) {
            const int32_t *row = idx + dsv_oracle_group_member(g, m, F, Hh, Ww, gf, gh, gw) * k;
            for (int64_t t = 0; t < k; ++t) count += in_centre[row[t]];
        }
        for (int64_t t = 0; t < k; ++t) in_centre[crow[t]] = 0;
    }
    free(in_centre);
    return count;
}

/* ---------------------------------------------------------------------------------------------
 * Predictor side (Sec. "Low-Rank based Sparsity Prediction", Sec. "Sparsity Profiling").
 *
 * Approximation loss of one head on a sample of n query rows (the paper samples queries at random to
 * bound the cost): with A = Q_s K^T [n, L] and Ahat = (Q_s Wq)(K Wk)^T [n, L],
 *     loss = 0.95 * CosLoss(Ahat, A) + 0.05 * NormLoss(Ahat, A).
 * Readings (the paper names the two terms and their weights only):
 *   CosLoss  = mean over the sampled queries of 1 - cos(ahat_i, a_i), the cosine between a query's
 *              approximate and true score ROWS (what ranks that query's keys);
 *   NormLoss = mean over all n * L entries of (ahat_ij - a_ij)^2;
 *   scores carry no softmax scale; projections are NOT rounded to the storage type here (the loss
 *   trains Wq, Wk in full precision; rounding belongs to the selection path).
 * Gradients of the loss with respect to Wq and Wk, by the chain rule written out:
 *     dAhat_ij = 0.95/n * ( -a_ij / (|ahat_i||a_i|) + <ahat_i, a_i> ahat_ij / (|ahat_i|^3 |a_i|) )
 *              + 0.05 * 2/(n L) * (ahat_ij - a_ij)
 *     dQlr = dAhat Klr,  dKlr = dAhat^T Qlr,  dWq = Q_s^T dQlr,  dWk = K^T dKlr.
 * Q_s [n, d], K [L, d], Wq, Wk [d, r].  Outputs: loss_parts[3] = {loss, CosLoss, NormLoss}, dWq, dWk [d, r].
 * ------------------------------------------------------------------------------------------- */
void dsv_oracle_predictor_loss(const float *Qs, const float *K, const float *Wq, const float *Wk, int64_t n,
                               int64_t L, int d, int r, double *loss_parts, double *dWq, double *dWk)
{
    double *Qlr = (double *)calloc((size_t)n * r, sizeof(double)), *Klr = (double *)calloc((size_t)L * r, sizeof(double));
    double *A = (double *)malloc((size_t)n * L * sizeof(double)), *Ah = (double *)malloc((size_t)n * L * sizeof(double));
    double *dA = (double *)malloc((size_t)n * L * sizeof(double));
    for (int64_t i = 0; i < n; ++i)
        for (int t = 0; t < r; ++t)
            for (int c = 0; c < d; ++c) Qlr[i * r + t] += (double)Qs[i * d + c] * (double)Wq[(int64_t)c * r + t];
    for (int64_t j = 0; j < L; ++j)
        for (int t = 0; t < r; ++t)
            for (int c = 0; c < d; ++c) Klr[j * r + t] += (double)K[j * d + c] * (double)Wk[(int64_t)c * r + t];
    double cos_loss = 0.0, norm_loss = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : cos_loss, norm_loss)
    for (int64_t i = 0; i < n; ++i) {
        double aa = 0.0, hh = 0.0, ah = 0.0, sq = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double a = 0.0, h = 0.0;
            for (int c = 0; c < d; ++c) a += (double)Qs[i * d + c] * (double)K[j * d + c];
            for (int t = 0; t < r; ++t) h += Qlr[i * r + t] * Klr[j * r + t];
            A[i * L + j] = a; Ah[i * L + j] = h;
            aa += a * a; hh += h * h; ah += a * h; sq += (h - a) * (h - a);
        }
        const double na = sqrt(aa), nh = sqrt(hh);
        cos_loss += (1.0 - ah / (na * nh)) / (double)n;
        norm_loss += sq / ((double)n * (double)L);
        for (int64_t j = 0; j < L; ++j)
            dA[i * L + j] = 0.95 / (double)n * (-A[i * L + j] / (nh * na) + ah * Ah[i * L + j] / (nh * nh * nh * na)) +
                            0.05 * 2.0 / ((double)n * (double)L) * (Ah[i * L + j] - A[i * L + j]);
    }
    loss_parts[0] = 0.95 * cos_loss + 0.05 * norm_loss;
    loss_parts[1] = cos_loss;
    loss_parts[2] = norm_loss;
    double *dQlr = (double *)calloc((size_t)n * r, sizeof(double)), *dKlr = (double *)calloc((size_t)L * r, sizeof(double));
    for (int64_t i = 0; i < n; ++i)
        for (int64_t j = 0; j < L; ++j)
            for (int t = 0; t < r; ++t) {
                dQlr[i * r + t] += dA[i * L + j] * Klr[j * r + t];
                dKlr[j * r + t] += dA[i * L + j] * Qlr[i * r + t];
            }
    for (int64_t e = 0; e < (int64_t)d * r; ++e) { dWq[e] = 0.0; dWk[e] = 0.0; }
    for (int64_t i = 0; i < n; ++i)
        for (int c = 0; c < d; ++c)
            for (int t = 0; t < r; ++t) dWq[(int64_t)c * r + t] += (double)Qs[i * d + c] * dQlr[i * r + t];
    for (int64_t j = 0; j < L; ++j)
        for (int c = 0; c < d; ++c)
            for (int t = 0; t < r; ++t) dWk[(int64_t)c * r + t] += (double)K[j * d + c] * dKlr[j * r + t];
    free(Qlr); free(Klr); free(A); free(Ah); free(dA); free(dQlr); free(dKlr);
}

/* Sparsity of one head measured on a sample of n query rows (Sec. "Exploiting Dynamic Sparsity": a
 * query's critical KV are the highest-probability keys that together hold `mass` (the paper: 90 %) of
 * its softmax; the head's sparsity is the mean fraction of NON-critical keys; Sec. "Sparsity Profiling":
 * measured on sampled queries).  For every sampled row: p = softmax(scale * q K^T) over all L keys, sorted
 * in descending order, c_i = the smallest count whose cumulative probability reaches `mass`.
 * Outputs: counts [n] (c_i), and the return value mean_i (1 - c_i / L). */
static int cmp_double_desc(const void *a, const void *b)
{
    const double x = *(const double *)a, y = *(const double *)b;
    return (x < y) - (x > y);
}

double dsv_oracle_profile_sparsity(const float *Qs, const float *K, int64_t n, int64_t L, int d, double scale,
                                   double mass, int64_t *counts)
{
    double total = 0.0;
#pragma omp parallel for schedule(dynamic, 1) reduction(+ : total)
    for (int64_t i = 0; i < n; ++i) {
        double *p = (double *)malloc((size_t)L * sizeof(double));
        double m = -INFINITY, z = 0.0;
        for (int64_t j = 0; j < L; ++j) {
            double acc = 0.0;
            for (int c = 0; c < d; ++c) acc += (double)Qs[i * d + c] * (double)K[j * d + c];
            p[j] = scale * acc;
            if (p[j] > m) m = p[j];
        }
        for (int64_t j = 0; j < L; ++j) z += exp(p[j] - m);
        for (int64_t j = 0; j < L; ++j) p[j] = exp(p[j] - m) / z;
        qsort(p, (size_t)L, sizeof(double), cmp_double_desc);
        double cum = 0.0;
        int64_t c = 0;
        while (c < L && cum < mass) cum += p[c++];
        counts[i] = c;
        total += 1.0 - (double)c / (double)L;
        free(p);
    }
    return total / (double)n;
}

/* Exponential moving average the profiler keeps per head and block: S_i = alpha P_i + (1 - alpha) S_{i-1}. */
double dsv_oracle_ema(double prev, double sample, double alpha) { return alpha * sample + (1.0 - alpha) * prev; }

int dsv_oracle_max_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}
