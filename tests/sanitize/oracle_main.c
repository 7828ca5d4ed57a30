/* Driver that runs every routine of the CPU oracle on small seeded inputs, edge shapes included, so that a
 * build with -fsanitize=address,undefined sees every loop and every index computation.  Besides the
 * sanitizers' own checks it asserts a few closed-form facts (they also hold in an unsanitized build). */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

double dsv_oracle_round(double x, int dtype);
void dsv_oracle_project(const float *X, const float *W, int64_t n, int d, int r, int dtype, float *out);
void dsv_oracle_scores(const float *Qlr, const float *Klr, int64_t nq, int64_t L, int r, double *S);
void dsv_oracle_topk_from_scores(const double *S, int64_t nq, int64_t L, int64_t k, int32_t *idx);
void dsv_oracle_lowrank_topk(const float *Q, const float *K, const float *Wq, const float *Wk, int64_t nq, int64_t L,
                             int d, int r, int64_t k, int dtype, int32_t *idx, float *Qlr_out, float *Klr_out,
                             double *S_out);
void dsv_oracle_sparse_fwd(const float *Q, const float *K, const float *V, const int32_t *idx, int64_t nq, int64_t L,
                           int d, int64_t k, double scale, double *O, double *lse, double *P);
void dsv_oracle_sparse_bwd(const float *Q, const float *K, const float *V, const int32_t *idx, const double *O,
                           const double *lse, const float *dO, int64_t L, int d, int64_t k, double scale, double *dQ,
                           double *dK, double *dV);
void dsv_oracle_sparse_bwd_dq_rows(const float *Q, const float *K, const float *V, const int32_t *idx,
                                   const double *O, const double *lse, const float *dO, int64_t nq, int d, int64_t k,
                                   double scale, double *dQ);
void dsv_oracle_sparse_bwd_dkdv_key(int32_t j, const float *Qs, const float *dOs, const double *Os,
                                    const double *lses, const int32_t *idxs, int64_t n, const float *K,
                                    const float *V, int d, int64_t k, double scale, double *dKj, double *dVj);
void dsv_oracle_dense_fwd(const float *Q, const float *K, const float *V, int64_t L, int d, double scale, double *O,
                          double *lse, double *P);
void dsv_oracle_dense_bwd(const float *Q, const float *K, const float *V, const float *dO, int64_t L, int d,
                          double scale, double *dQ, double *dK, double *dV);
int dsv_oracle_max_threads(void);
int64_t dsv_oracle_group_member(int64_t g, int m, int F, int Hh, int Ww, int gf, int gh, int gw);
int dsv_oracle_group_centre(int gf, int gh, int gw);
void dsv_oracle_lowrank_topk_grouped(const float *Q, const float *K, const float *Wq, const float *Wk, int F, int Hh, int Ww,
                                     int gf, int gh, int gw, int d, int r, int64_t k, int dtype, int32_t *idx_g);
void dsv_oracle_group_expand_idx(const int32_t *idx_g, int F, int Hh, int Ww, int gf, int gh, int gw, int64_t k, int32_t *idx);
int64_t dsv_oracle_group_overlap(const int32_t *idx, int F, int Hh, int Ww, int gf, int gh, int gw, int64_t k);
void dsv_oracle_sparse_fwd_grouped(const float *Q, const float *K, const float *V, const int32_t *idx_g, int F, int Hh, int Ww,
                                   int gf, int gh, int gw, int d, int64_t k, double scale, double *O, double *lse);
void dsv_oracle_sparse_bwd_grouped(const float *Q, const float *K, const float *V, const int32_t *idx_g, const float *dO, int F,
                                   int Hh, int Ww, int gf, int gh, int gw, int d, int64_t k, double scale, double *dQ, double *dK,
                                   double *dV);
void dsv_oracle_predictor_loss(const float *Qs, const float *K, const float *Wq, const float *Wk, int64_t n, int64_t L, int d,
                               int r, double *loss_parts, double *dWq, double *dWk);
double dsv_oracle_profile_sparsity(const float *Qs, const float *K, int64_t n, int64_t L, int d, double scale, double mass,
                                   int64_t *counts);
double dsv_oracle_ema(double prev, double sample, double alpha);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static float rnd(void)
{
    state ^= state << 13; state ^= state >> 7; state ^= state << 17;
    return (float)((double)(state >> 11) / 9007199254740992.0 * 2.0 - 1.0);
}
static float *fvec(size_t n)
{
    float *p = (float *)malloc((n ? n : 1) * sizeof(float));
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); exit(1); } } while (0)

static void one_shape(int64_t L, int d, int r, int64_t k, int dtype)
{
    float *Q = fvec((size_t)L * d), *K = fvec((size_t)L * d), *V = fvec((size_t)L * d), *dO = fvec((size_t)L * d);
    float *Wq = fvec((size_t)d * r), *Wk = fvec((size_t)d * r);
    int32_t *idx = (int32_t *)malloc((size_t)L * k * sizeof(int32_t));
    float *Qlr = (float *)malloc((size_t)L * r * sizeof(float)), *Klr = (float *)malloc((size_t)L * r * sizeof(float));
    double *S = (double *)malloc((size_t)L * L * sizeof(double));
    dsv_oracle_lowrank_topk(Q, K, Wq, Wk, L, L, d, r, k, dtype, idx, Qlr, Klr, S);
    dsv_oracle_lowrank_topk(Q, K, Wq, Wk, L, L, d, r, k, dtype, idx, NULL, NULL, NULL);
    for (int64_t i = 0; i < L; ++i)
        for (int64_t t = 0; t < k; ++t) {
            CHECK(idx[i * k + t] >= 0 && idx[i * k + t] < L);
            if (t) CHECK(idx[i * k + t] > idx[i * k + t - 1]);
        }
    double *O = (double *)malloc((size_t)L * d * sizeof(double)), *lse = (double *)malloc((size_t)L * sizeof(double));
    double *P = (double *)malloc((size_t)L * k * sizeof(double));
    dsv_oracle_sparse_fwd(Q, K, V, idx, L, L, d, k, 0.25, O, lse, P);
    for (int64_t i = 0; i < L; ++i) {
        double s = 0.0;
        for (int64_t t = 0; t < k; ++t) s += P[i * k + t];
        CHECK(fabs(s - 1.0) < 1e-12);
    }
    double *dQ = (double *)malloc((size_t)L * d * sizeof(double)), *dK = (double *)malloc((size_t)L * d * sizeof(double));
    double *dV = (double *)malloc((size_t)L * d * sizeof(double)), *dQ2 = (double *)malloc((size_t)L * d * sizeof(double));
    dsv_oracle_sparse_bwd(Q, K, V, idx, O, lse, dO, L, d, k, 0.25, dQ, dK, dV);
    dsv_oracle_sparse_bwd_dq_rows(Q, K, V, idx, O, lse, dO, L, d, k, 0.25, dQ2);
    for (int64_t e = 0; e < L * d; ++e) CHECK(fabs(dQ[e] - dQ2[e]) <= 1e-12 * (1.0 + fabs(dQ[e])));
    /* one key from the queries that hold it */
    const int32_t j = idx[0];
    int64_t n = 0;
    float *Qs = (float *)malloc((size_t)L * d * sizeof(float)), *Gs = (float *)malloc((size_t)L * d * sizeof(float));
    double *Os = (double *)malloc((size_t)L * d * sizeof(double)), *ls = (double *)malloc((size_t)L * sizeof(double));
    int32_t *is = (int32_t *)malloc((size_t)L * k * sizeof(int32_t));
    for (int64_t i = 0; i < L; ++i) {
        int has = 0;
        for (int64_t t = 0; t < k; ++t) has |= idx[i * k + t] == j;
        if (!has) continue;
        for (int c = 0; c < d; ++c) { Qs[n * d + c] = Q[i * d + c]; Gs[n * d + c] = dO[i * d + c]; Os[n * d + c] = O[i * d + c]; }
        for (int64_t t = 0; t < k; ++t) is[n * k + t] = idx[i * k + t];
        ls[n++] = lse[i];
    }
    double *dKj = (double *)malloc((size_t)d * sizeof(double)), *dVj = (double *)malloc((size_t)d * sizeof(double));
    dsv_oracle_sparse_bwd_dkdv_key(j, Qs, Gs, Os, ls, is, n, K, V, d, k, 0.25, dKj, dVj);
    for (int c = 0; c < d; ++c) {
        CHECK(fabs(dKj[c] - dK[(int64_t)j * d + c]) <= 1e-10 * (1.0 + fabs(dKj[c])));
        CHECK(fabs(dVj[c] - dV[(int64_t)j * d + c]) <= 1e-10 * (1.0 + fabs(dVj[c])));
    }
    /* dense routines, and the k = L limit */
    double *Od = (double *)malloc((size_t)L * d * sizeof(double)), *lsd = (double *)malloc((size_t)L * sizeof(double));
    double *Pd = (double *)malloc((size_t)L * L * sizeof(double));
    dsv_oracle_dense_fwd(Q, K, V, L, d, 0.25, Od, lsd, Pd);
    dsv_oracle_dense_fwd(Q, K, V, L, d, 0.25, Od, lsd, NULL);
    dsv_oracle_dense_bwd(Q, K, V, dO, L, d, 0.25, dQ, dK, dV);
    if (k == L)
        for (int64_t e = 0; e < L * d; ++e) CHECK(fabs(O[e] - Od[e]) < 1e-11);
    free(Q); free(K); free(V); free(dO); free(Wq); free(Wk); free(idx); free(Qlr); free(Klr); free(S); free(O);
    free(lse); free(P); free(dQ); free(dK); free(dV); free(dQ2); free(Qs); free(Gs); free(Os); free(ls); free(is);
    free(dKj); free(dVj); free(Od); free(lsd); free(Pd);
}

/* query grouping, group-size profiling and the predictor side on one small grid */
static void grouped_shape(int F, int Hh, int Ww, int gf, int gh, int gw, int d, int r, int64_t k)
{
    const int64_t L = (int64_t)F * Hh * Ww;
    const int G = gf * gh * gw;
    float *Q = fvec((size_t)L * d), *K = fvec((size_t)L * d), *V = fvec((size_t)L * d), *dO = fvec((size_t)L * d);
    float *Wq = fvec((size_t)d * r), *Wk = fvec((size_t)d * r);
    int32_t *idx_g = (int32_t *)malloc((size_t)(L / G) * k * sizeof(int32_t));
    int32_t *idx = (int32_t *)malloc((size_t)L * k * sizeof(int32_t));
    dsv_oracle_lowrank_topk_grouped(Q, K, Wq, Wk, F, Hh, Ww, gf, gh, gw, d, r, k, 1, idx_g);
    dsv_oracle_group_expand_idx(idx_g, F, Hh, Ww, gf, gh, gw, k, idx);
    CHECK(dsv_oracle_group_overlap(idx, F, Hh, Ww, gf, gh, gw, k) == L * k);     /* every member uses its centre's row */
    CHECK(dsv_oracle_group_overlap(idx, F, Hh, Ww, gf + 1, gh, gw, k) == -1 || F % (gf + 1) == 0);
    const int c = dsv_oracle_group_centre(gf, gh, gw);
    CHECK(c >= 0 && c < G && dsv_oracle_group_member(L / G - 1, G - 1, F, Hh, Ww, gf, gh, gw) == L - 1);
    double *O = (double *)malloc((size_t)L * d * sizeof(double)), *lse = (double *)malloc((size_t)L * sizeof(double));
    double *dQ = (double *)malloc((size_t)L * d * sizeof(double)), *dK = (double *)malloc((size_t)L * d * sizeof(double));
    double *dV = (double *)malloc((size_t)L * d * sizeof(double));
    dsv_oracle_sparse_fwd_grouped(Q, K, V, idx_g, F, Hh, Ww, gf, gh, gw, d, k, 0.25, O, lse);
    dsv_oracle_sparse_bwd_grouped(Q, K, V, idx_g, dO, F, Hh, Ww, gf, gh, gw, d, k, 0.25, dQ, dK, dV);
    double parts[3];
    double *dWq = (double *)malloc((size_t)d * r * sizeof(double)), *dWk = (double *)malloc((size_t)d * r * sizeof(double));
    const int64_t n = L / 3 + 1;
    dsv_oracle_predictor_loss(Q, K, Wq, Wk, n, L, d, r, parts, dWq, dWk);
    CHECK(parts[1] >= 0.0 && parts[1] <= 2.0 && parts[2] >= 0.0 && fabs(parts[0] - (0.95 * parts[1] + 0.05 * parts[2])) < 1e-12);
    int64_t *counts = (int64_t *)malloc((size_t)n * sizeof(int64_t));
    const double sp = dsv_oracle_profile_sparsity(Q, K, n, L, d, 0.25, 0.9, counts);
    CHECK(sp >= 0.0 && sp < 1.0);
    for (int64_t i = 0; i < n; ++i) CHECK(counts[i] >= 1 && counts[i] <= L);
    CHECK(dsv_oracle_ema(0.5, 1.0, 0.1) == 0.1 * 1.0 + 0.9 * 0.5);
    free(Q); free(K); free(V); free(dO); free(Wq); free(Wk); free(idx_g); free(idx); free(O); free(lse); free(dQ); free(dK);
    free(dV); free(dWq); free(dWk); free(counts);
}

int main(void)
{
    CHECK(dsv_oracle_round(1.0 + 1.0 / 256.0, 1) == 1.0);          /* bf16 tie to even */
    CHECK(dsv_oracle_round(1.0 + 3.0 / 256.0, 1) == 1.0 + 1.0 / 64.0);
    CHECK(dsv_oracle_round(1e-45, 0) == ldexp(1.0, -149));           /* smallest fp32 subnormal */
    CHECK(dsv_oracle_round(0.0, 1) == 0.0);
    CHECK(dsv_oracle_max_threads() >= 1);
    one_shape(1, 8, 2, 1, 0);        /* a single token */
    one_shape(7, 4, 2, 1, 1);        /* k = 1 */
    one_shape(33, 16, 4, 33, 1);     /* k = L */
    one_shape(65, 64, 16, 9, 0);
    one_shape(130, 128, 32, 64, 1);
    grouped_shape(2, 4, 6, 2, 2, 2, 16, 4, 7);
    grouped_shape(3, 2, 5, 1, 1, 1, 8, 2, 30);     /* unit cube, k = L */
    grouped_shape(2, 6, 3, 1, 3, 3, 32, 8, 1);     /* G = 9, k = 1 */
    printf("oracle sanitizer run ok\n");
    return 0;
}
