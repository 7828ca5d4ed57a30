// Predictor side (paper Sec. "Low-Rank based Sparsity Prediction"): the approximation loss
//     0.95 * CosLoss + 0.05 * NormLoss   between  Ahat = (Q_s Wq)(K Wk)^T  and  A = Q_s K^T
// on a sample of query rows, and its gradients for Wq and Wk -- without ever forming a row of A or Ahat.
//
// Every quantity the loss needs is a quadratic form in the key Gram matrix M = K^T K [d, d]:
//     |a_i|^2 = q_i^T M q_i,   <ahat_i, a_i> = qlr_i^T (Wk^T M q_i),   |ahat_i|^2 = qlr_i^T (Wk^T M Wk) qlr_i,
//     sum_j (ahat_ij - a_ij)^2 = |ahat_i|^2 - 2 <ahat_i, a_i> + |a_i|^2,
// and with dAhat_i = ca_i a_i + ch_i ahat_i (the chain rule of the two terms; coefficients below)
//     dWq = Q_s^T G,           G_i  = ca_i (Wk^T M q_i) + ch_i (Wk^T M Wk) qlr_i        (= dAhat_i Klr)
//     dWk = M (N1 + Wk N2),    N1 = sum_i ca_i q_i qlr_i^T,  N2 = sum_i ch_i qlr_i qlr_i^T   (= K^T dAhat^T Qlr).
// So the only pass over all L keys is the Gram matrix (K is read once: HBM-bound); the rest is small dense
// algebra on [d, d], [d, r] and the n sampled rows, done in fp64 (the norm term cancels to a small difference
// of large sums when the predictor is good).  The paper's point -- no [n, L] intermediate is stored -- holds in
// the strongest form: none is computed.
#include <algorithm>

#include "common.h"

namespace dsv {

// ---- M = K^T K, partial sums over token blocks ---------------------------------------------------------
// grid (nblk, B*H); block 256 = 16 x 16 threads, thread (ty, tx) owns the entries of M at rows ty + 16 a,
// columns tx + 16 b (a, b < D/16: conflict-free LDS reads); tokens pass through LDS 32 at a time as fp32.
template <typename T, int D>
__global__ __launch_bounds__(256) void gram_partial_kernel(const T *__restrict__ K, int L, int tok_per_block,
                                                           float *__restrict__ part)
{
    constexpr int S = D / 16;
    __shared__ float tile[32][D + 4];
    const int bh = blockIdx.y;
    const int t0 = blockIdx.x * tok_per_block, t1 = min(t0 + tok_per_block, L);
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;
    const T *Kh = K + (int64_t)bh * L * D;
    float acc[S][S];
#pragma unroll
    for (int a = 0; a < S; ++a)
#pragma unroll
        for (int b = 0; b < S; ++b) acc[a][b] = 0.f;
    for (int tb = t0; tb < t1; tb += 32) {
        for (int e = threadIdx.x; e < 32 * D; e += 256) {
            const int t = e / D, c = e % D;
            tile[t][c] = tb + t < t1 ? to_f32<T>(Kh[(int64_t)(tb + t) * D + c]) : 0.f;
        }
        __syncthreads();
#pragma unroll 4
        for (int t = 0; t < 32; ++t) {
            float ra[S], rb[S];
#pragma unroll
            for (int a = 0; a < S; ++a) { ra[a] = tile[t][ty + 16 * a]; rb[a] = tile[t][tx + 16 * a]; }
#pragma unroll
            for (int a = 0; a < S; ++a)
#pragma unroll
                for (int b = 0; b < S; ++b) acc[a][b] = fmaf(ra[a], rb[b], acc[a][b]);
        }
        __syncthreads();
    }
    float *out = part + ((int64_t)bh * gridDim.x + blockIdx.x) * D * D;
#pragma unroll
    for (int a = 0; a < S; ++a)
#pragma unroll
        for (int b = 0; b < S; ++b) out[(ty + 16 * a) * D + tx + 16 * b] = acc[a][b];
}

// M[bh] = sum of the partials (fp64); then T1 = M Wk [D, R] and T2 = Wk^T T1 [R, R].  One block per head.
template <typename T>
__global__ __launch_bounds__(256) void gram_finish_kernel(const float *__restrict__ part, int nblk, const T *__restrict__ Wk,
                                                          int H, int D, int R, double *__restrict__ M,
                                                          double *__restrict__ T1, double *__restrict__ T2)
{
    const int bh = blockIdx.x;
    const T *W = Wk + (int64_t)(bh % H) * D * R;
    double *Mh = M + (int64_t)bh * D * D, *T1h = T1 + (int64_t)bh * D * R, *T2h = T2 + (int64_t)bh * R * R;
    for (int e = threadIdx.x; e < D * D; e += 256) {
        double s = 0.0;
        for (int b = 0; b < nblk; ++b) s += (double)part[((int64_t)bh * nblk + b) * D * D + e];
        Mh[e] = s;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < D * R; e += 256) {
        const int c = e / R, t = e % R;
        double s = 0.0;
        for (int c2 = 0; c2 < D; ++c2) s += Mh[c * D + c2] * (double)to_f32<T>(W[c2 * R + t]);
        T1h[e] = s;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < R * R; e += 256) {
        const int a = e / R, b = e % R;
        double s = 0.0;
        for (int c = 0; c < D; ++c) s += (double)to_f32<T>(W[c * R + a]) * T1h[c * R + b];
        T2h[e] = s;
    }
}

// ---- per sampled row ------------------------------------------------------------------------------------
// One wave per (head, sampled row).  Writes, per row: qlr [R], G [R] (= dAhat_i Klr), CA = ca_i qlr, CH = ch_i qlr,
// and the row's loss terms {1 - cos_i, sum_j (ahat_ij - a_ij)^2}.
//   ca_i = -0.95 / (n |ahat_i| |a_i|) - 0.1 / (n L),   ch_i = 0.95 <ahat_i, a_i> / (n |ahat_i|^3 |a_i|) + 0.1 / (n L)
template <typename T>
__global__ __launch_bounds__(256) void predictor_rows_kernel(const T *__restrict__ Q, const T *__restrict__ Wq,
                                                             const int32_t *__restrict__ rows, int n, int L, int H, int D,
                                                             int R, const double *__restrict__ M,
                                                             const double *__restrict__ T1, const double *__restrict__ T2,
                                                             double *__restrict__ qlr_out, double *__restrict__ g_out,
                                                             double *__restrict__ ca_out, double *__restrict__ ch_out,
                                                             double *__restrict__ terms)
{
    __shared__ double sh_all[4][128 + 64 + 64 + 64];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + wave;
    const int bh = blockIdx.y;
    if (i >= n) return;  // whole wave
    double *q = sh_all[wave], *ql = q + 128, *v = ql + 64, *w = v + 64;
    const int row = min(max(rows[i], 0), L - 1);
    const T *qrow = Q + ((int64_t)bh * L + row) * D;
    const T *Wh = Wq + (int64_t)(bh % H) * D * R;
    const double *Mh = M + (int64_t)bh * D * D, *T1h = T1 + (int64_t)bh * D * R, *T2h = T2 + (int64_t)bh * R * R;
    for (int c = lane; c < D; c += 64) q[c] = (double)to_f32<T>(qrow[c]);
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // aa = q^T M q
    double aa = 0.0;
    for (int c = lane; c < D; c += 64) {
        double u = 0.0;
        for (int c2 = 0; c2 < D; ++c2) u += Mh[c2 * D + c] * q[c2];  // M is symmetric: column c, coalesced
        aa += q[c] * u;
    }
    for (int o = 32; o; o >>= 1) aa += __shfl_xor(aa, o);
    // qlr = Wq^T q,  v = T1^T q
    for (int t = lane; t < R; t += 64) {
        double a = 0.0, b = 0.0;
        for (int c = 0; c < D; ++c) { a += (double)to_f32<T>(Wh[c * R + t]) * q[c]; b += T1h[c * R + t] * q[c]; }
        ql[t] = a;
        v[t] = b;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    double ah = 0.0, hh = 0.0;
    for (int t = lane; t < R; t += 64) {
        double ww = 0.0;
        for (int t2 = 0; t2 < R; ++t2) ww += T2h[t2 * R + t] * ql[t2];  // T2 is symmetric
        w[t] = ww;
        ah += ql[t] * v[t];
        hh += ql[t] * ww;
    }
    for (int o = 32; o; o >>= 1) { ah += __shfl_xor(ah, o); hh += __shfl_xor(hh, o); }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront"); __builtin_amdgcn_wave_barrier(); __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const double na = sqrt(aa), nh = sqrt(hh);
    const double ca = -0.95 / ((double)n * nh * na) - 0.1 / ((double)n * (double)L);
    const double ch = 0.95 * ah / ((double)n * nh * nh * nh * na) + 0.1 / ((double)n * (double)L);
    const int64_t o = ((int64_t)bh * n + i) * R;
    for (int t = lane; t < R; t += 64) {
        qlr_out[o + t] = ql[t];
        g_out[o + t] = ca * v[t] + ch * w[t];
        ca_out[o + t] = ca * ql[t];
        ch_out[o + t] = ch * ql[t];
    }
    if (lane == 0) {
        terms[((int64_t)bh * n + i) * 2 + 0] = 1.0 - ah / (na * nh);
        terms[((int64_t)bh * n + i) * 2 + 1] = hh - 2.0 * ah + aa;
    }
}

// ---- sums over the sampled rows ---------------------------------------------------------------------------
// dWq = Q_s^T G [D, R],  N1 = Q_s^T CA [D, R],  N2 = Qlr^T CH [R, R]: every block takes 32 sampled rows (their Q
// rows and per-row vectors staged in LDS) and writes its partial sums; predictor_finish_kernel adds the partials
// in block order (deterministic).
constexpr int kAccRows = 32;
template <typename T>
__global__ __launch_bounds__(256) void predictor_accum_kernel(const T *__restrict__ Q, const int32_t *__restrict__ rows,
                                                              int n, int L, int D, int R, const double *__restrict__ qlr,
                                                              const double *__restrict__ g, const double *__restrict__ ca,
                                                              const double *__restrict__ ch, double *__restrict__ p_dwq,
                                                              double *__restrict__ p_n1, double *__restrict__ p_n2)
{
    __shared__ float xq[kAccRows][128];
    __shared__ double yg[kAccRows][64], yca[kAccRows][64], ych[kAccRows][64], xl[kAccRows][64];
    const int bh = blockIdx.y, chunk = blockIdx.x;
    const int i0 = chunk * kAccRows, ni = min(kAccRows, n - i0);
    for (int e = threadIdx.x; e < kAccRows * D; e += 256) {
        const int i = e / D, c = e % D;
        xq[i][c] = i < ni ? to_f32<T>(Q[((int64_t)bh * L + min(max(rows[i0 + i], 0), L - 1)) * D + c]) : 0.f;
    }
    for (int e = threadIdx.x; e < kAccRows * R; e += 256) {
        const int i = e / R, t = e % R;
        const int64_t o = ((int64_t)bh * n + i0 + i) * R + t;
        yg[i][t] = i < ni ? g[o] : 0.0;
        yca[i][t] = i < ni ? ca[o] : 0.0;
        ych[i][t] = i < ni ? ch[o] : 0.0;
        xl[i][t] = i < ni ? qlr[o] : 0.0;
    }
    __syncthreads();
    const int64_t pb = (int64_t)bh * gridDim.x + chunk;
    for (int e = threadIdx.x; e < D * R; e += 256) {
        const int c = e / R, t = e % R;
        double s1 = 0.0, s2 = 0.0;
        for (int i = 0; i < kAccRows; ++i) { s1 += (double)xq[i][c] * yg[i][t]; s2 += (double)xq[i][c] * yca[i][t]; }
        p_dwq[pb * D * R + e] = s1;
        p_n1[pb * D * R + e] = s2;
    }
    for (int e = threadIdx.x; e < R * R; e += 256) {
        const int a = e / R, t = e % R;
        double s = 0.0;
        for (int i = 0; i < kAccRows; ++i) s += xl[i][a] * ych[i][t];
        p_n2[pb * R * R + e] = s;
    }
}

// dWk = M (N1 + Wk N2), dWq and N1, N2 from the blocks' partials; loss = {0.95 cos + 0.05 norm, cos, norm}.  One block per head.
template <typename T>
__global__ __launch_bounds__(256) void predictor_finish_kernel(const double *__restrict__ M, const T *__restrict__ Wk,
                                                               const double *__restrict__ p_dwq, const double *__restrict__ p_n1,
                                                               const double *__restrict__ p_n2, int nchunk,
                                                               const double *__restrict__ terms, int n, int L, int H, int D,
                                                               int R, float *__restrict__ loss, float *__restrict__ dWq,
                                                               float *__restrict__ dWk)
{
    extern __shared__ double sh[];  // P [D, R] = N1 + Wk N2, then N2 [R, R], then 2 x 256 reduction slots
    double *P = sh, *N2 = sh + D * R, *red = N2 + R * R;
    const int bh = blockIdx.x;
    const T *W = Wk + (int64_t)(bh % H) * D * R;
    for (int e = threadIdx.x; e < R * R; e += 256) {
        double s = 0.0;
        for (int c = 0; c < nchunk; ++c) s += p_n2[((int64_t)bh * nchunk + c) * R * R + e];
        N2[e] = s;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < D * R; e += 256) {
        const int c = e / R, t = e % R;
        double s = 0.0, q = 0.0;
        for (int k = 0; k < nchunk; ++k) {
            s += p_n1[((int64_t)bh * nchunk + k) * D * R + e];
            q += p_dwq[((int64_t)bh * nchunk + k) * D * R + e];
        }
        for (int t2 = 0; t2 < R; ++t2) s += (double)to_f32<T>(W[c * R + t2]) * N2[t2 * R + t];
        P[e] = s;
        dWq[(int64_t)bh * D * R + e] = (float)q;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < D * R; e += 256) {
        const int c = e / R, t = e % R;
        double s = 0.0;
        for (int c2 = 0; c2 < D; ++c2) s += M[(int64_t)bh * D * D + c * D + c2] * P[c2 * R + t];
        dWk[(int64_t)bh * D * R + e] = (float)s;
    }
    double c = 0.0, m = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) { c += terms[((int64_t)bh * n + i) * 2]; m += terms[((int64_t)bh * n + i) * 2 + 1]; }
    red[threadIdx.x] = c;
    red[256 + threadIdx.x] = m;
    __syncthreads();
    for (int step = 128; step; step >>= 1) {
        if ((int)threadIdx.x < step) { red[threadIdx.x] += red[threadIdx.x + step]; red[256 + threadIdx.x] += red[256 + threadIdx.x + step]; }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        c = red[0] / (double)n;
        m = red[256] / ((double)n * (double)L);
        loss[bh * 3 + 0] = (float)(0.95 * c + 0.05 * m);
        loss[bh * 3 + 1] = (float)c;
        loss[bh * 3 + 2] = (float)m;
    }
}

// ------------------------------------------------------------------------------------ host
PredictorLayout predictor_layout(const dsv_problem &p, int n)
{
    const size_t nbh = (size_t)p.B * p.H, D = p.d, R = p.r;
    PredictorLayout w{};
    w.tok_per_block = 1024;
    w.nblk = (p.L + w.tok_per_block - 1) / w.tok_per_block;
    size_t o = 0;
    w.part = o; o = align_up(o + nbh * w.nblk * D * D * 4, 256);
    w.M = o; o = align_up(o + nbh * D * D * 8, 256);
    w.T1 = o; o = align_up(o + nbh * D * R * 8, 256);
    w.T2 = o; o = align_up(o + nbh * R * R * 8, 256);
    w.qlr = o; o = align_up(o + nbh * n * R * 8, 256);
    w.g = o; o = align_up(o + nbh * n * R * 8, 256);
    w.ca = o; o = align_up(o + nbh * n * R * 8, 256);
    w.ch = o; o = align_up(o + nbh * n * R * 8, 256);
    w.terms = o; o = align_up(o + nbh * n * 2 * 8, 256);
    w.nchunk = (n + 31) / 32;   // kAccRows sampled rows per partial sum
    w.dwq = o; o = align_up(o + nbh * w.nchunk * D * R * 8, 256);
    w.n1 = o; o = align_up(o + nbh * w.nchunk * D * R * 8, 256);
    w.n2 = o; o = align_up(o + nbh * w.nchunk * R * R * 8, 256);
    w.total = o;
    return w;
}

template <typename T>
static dsv_status predictor_t(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                              const int32_t *rows, int n, float *loss, float *dWq, float *dWk, char *ws,
                              const PredictorLayout &w, hipStream_t st)
{
    const int nbh = p.B * p.H, D = p.d, R = p.r;
    float *part = reinterpret_cast<float *>(ws + w.part);
    double *M = reinterpret_cast<double *>(ws + w.M), *T1 = reinterpret_cast<double *>(ws + w.T1);
    double *T2 = reinterpret_cast<double *>(ws + w.T2), *qlr = reinterpret_cast<double *>(ws + w.qlr);
    double *g = reinterpret_cast<double *>(ws + w.g), *ca = reinterpret_cast<double *>(ws + w.ca);
    double *ch = reinterpret_cast<double *>(ws + w.ch), *terms = reinterpret_cast<double *>(ws + w.terms);
    double *dwq = reinterpret_cast<double *>(ws + w.dwq), *n1 = reinterpret_cast<double *>(ws + w.n1);
    double *n2 = reinterpret_cast<double *>(ws + w.n2);
    if (D == 128)
        hipLaunchKernelGGL((gram_partial_kernel<T, 128>), dim3(w.nblk, nbh), dim3(256), 0, st, (const T *)K, p.L, w.tok_per_block, part);
    else
        hipLaunchKernelGGL((gram_partial_kernel<T, 64>), dim3(w.nblk, nbh), dim3(256), 0, st, (const T *)K, p.L, w.tok_per_block, part);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL((gram_finish_kernel<T>), dim3(nbh), dim3(256), 0, st, part, w.nblk, (const T *)Wk, p.H, D, R, M, T1, T2);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL((predictor_rows_kernel<T>), dim3((n + 3) / 4, nbh), dim3(256), 0, st, (const T *)Q, (const T *)Wq, rows, n,
                       p.L, p.H, D, R, M, T1, T2, qlr, g, ca, ch, terms);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL((predictor_accum_kernel<T>), dim3(w.nchunk, nbh), dim3(256), 0, st, (const T *)Q, rows, n, p.L, D, R, qlr, g,
                       ca, ch, dwq, n1, n2);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL((predictor_finish_kernel<T>), dim3(nbh), dim3(256), (size_t)(D * R + R * R + 512) * 8, st, M, (const T *)Wk,
                       dwq, n1, n2, w.nchunk, terms, n, p.L, p.H, D, R, loss, dWq, dWk);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_predictor_loss(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                                 const int32_t *rows, int n, float *loss, float *dWq, float *dWk, char *ws,
                                 const PredictorLayout &w, hipStream_t st)
{
    if (p.dtype == DSV_BF16) return predictor_t<bf16_t>(p, Q, K, Wq, Wk, rows, n, loss, dWq, dWk, ws, w, st);
    return predictor_t<float>(p, Q, K, Wq, Wk, rows, n, loss, dWq, dWk, ws, w, st);
}

}  // namespace dsv
