// Stage 2: exact softmax attention over the selected KV only, forward and backward
// (paper Sec. "Sparse Attention with Query Grouping", per-query form; attention formula of
// Sec. "Various Self-Attention Paradigms").
//
// Work layout shared by the kernels here: a group of 16 lanes (one DPP row) owns one query row;
// lane s of the group holds channels [s*CH, (s+1)*CH) of every [d]-vector, CH = d/16, so one
// wave-wide load instruction fetches four whole K (or V) rows as four contiguous segments.
// Dot products are reduced inside the row with DPP rotations.  A wave handles 4 queries, a block
// 16 consecutive queries of one head.
#include <algorithm>

#include "common.h"

namespace dsv {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ------------------------------------------------------------------------------------ forward
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_fwd_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                         const T *__restrict__ V, const int32_t *__restrict__ idx,
                                                         T *__restrict__ O, float *__restrict__ lse, int L,
                                                         float scale, HeadTable tab)
{
    constexpr int CH = D / 16;
    constexpr int U = 4;  // keys in flight per group
    typedef RowChunk<T, CH> Chunk;
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t iq = (int64_t)blockIdx.x * 16 + wave * 4 + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Kb = K + head_base + s * CH;
    const T *Vb = V + head_base + s * CH;
    const int32_t *row = idx + tab.off[slot] + i * k;

    const Chunk q = load_chunk<T, CH>(Q + head_base + i * D + s * CH);
    const float c2 = scale * kLog2e;  // logits are kept in the log2 domain

    float m = -INFINITY, l = 0.f;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;

    for (int t0 = 0; t0 < k; t0 += U) {
        int j[U];
        Chunk kc[U], vc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) j[u] = row[min(t0 + u, k - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            kc[u] = load_chunk<T, CH>(Kb + (int64_t)j[u] * D);
            vc[u] = load_chunk<T, CH>(Vb + (int64_t)j[u] * D);
        }
        float sc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) sc[u] = dot_chunk<T, CH>(q, kc[u]);
#pragma unroll
        for (int u = 0; u < U; ++u) sc[u] = row16_sum(sc[u]) * c2;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (t0 + u >= k) sc[u] = -INFINITY;
        float mnew = m;
#pragma unroll
        for (int u = 0; u < U; ++u) mnew = fmaxf(mnew, sc[u]);
        const float corr = exp2f(m - mnew);  // first block: exp2(-inf) = 0
        m = mnew;
        l *= corr;
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[c] *= corr;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float pu = exp2f(sc[u] - mnew);
            l += pu;
            float vf[CH];
            unpack_chunk<T, CH>(vc[u], vf);
#pragma unroll
            for (int c = 0; c < CH; ++c) acc[c] = fmaf(pu, vf[c], acc[c]);
        }
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] *= inv;
    if (live) {
        store_chunk<T, CH>(O + head_base + i * D + s * CH, acc);
        if (s == 0) lse[(int64_t)bh * L + i] = (m + log2f(l)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------ backward
// The backward runs as two gather passes with no floating-point atomics:
//   dq pass    query-major over idx: dQ and the row term Delta_i;
//   dkdv pass  key-major over the transposed index (for each key, the queries that selected it):
//              dK and dV, each output row owned by one lane group.
// Delta_i = dO_i . O_i equals sum_j p_ij (dO_i . v_j) over the selected keys; the dq pass forms it
// from that sum in fp32 instead of from the stored (storage-type rounded) O, and expands
//   dQ_i = scale * ( sum_j p_ij dP_ij k_j  -  Delta_i * sum_j p_ij k_j ),   dP_ij = dO_i . v_j,
// so one sweep over the row yields both.  Delta is kept for the dkdv pass.
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dq_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                            const T *__restrict__ V,
                                                            const int32_t *__restrict__ idx,
                                                            const float *__restrict__ lse, const T *__restrict__ dO,
                                                            T *__restrict__ dQ, float *__restrict__ delta_out, int L,
                                                            float scale, HeadTable tab)
{
    constexpr int CH = D / 16;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t iq = (int64_t)blockIdx.x * 16 + wave * 4 + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Kb = K + head_base + s * CH;
    const T *Vb = V + head_base + s * CH;
    const int32_t *row = idx + tab.off[slot] + i * k;

    const Chunk q = load_chunk<T, CH>(Q + head_base + i * D + s * CH);
    const Chunk go = load_chunk<T, CH>(dO + head_base + i * D + s * CH);
    const float c2 = scale * kLog2e;
    const float lse2 = lse[(int64_t)bh * L + i] * kLog2e;

    float a[CH], bsum[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { a[c] = 0.f; bsum[c] = 0.f; }
    float delta = 0.f;

    for (int t0 = 0; t0 < k; t0 += U) {
        int j[U];
        Chunk kc[U], vc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) j[u] = row[min(t0 + u, k - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            kc[u] = load_chunk<T, CH>(Kb + (int64_t)j[u] * D);
            vc[u] = load_chunk<T, CH>(Vb + (int64_t)j[u] * D);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float sc = row16_sum(dot_chunk<T, CH>(q, kc[u]));
            const float dp = row16_sum(dot_chunk<T, CH>(go, vc[u]));
            const float p = (t0 + u < k) ? exp2f(sc * c2 - lse2) : 0.f;
            const float pdp = p * dp;
            delta += pdp;
            float kf[CH];
            unpack_chunk<T, CH>(kc[u], kf);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                a[c] = fmaf(pdp, kf[c], a[c]);
                bsum[c] = fmaf(p, kf[c], bsum[c]);
            }
        }
    }
    if (live) {
        float dq[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) dq[c] = scale * (a[c] - delta * bsum[c]);
        store_chunk<T, CH>(dQ + head_base + i * D + s * CH, dq);
        if (s == 0) delta_out[(int64_t)bh * L + i] = delta;
    }
}

// ---- transposed index: for every key, the list of queries whose row holds it ----------------
// Counting sort by key.  cnt[bh, j] = number of rows holding j; col[bh, j] = exclusive prefix sum;
// the fill pass appends each query to its keys' lists through an atomic cursor, so the order
// inside a list is not fixed (only the fp32 summation order of dK, dV depends on it).
__global__ __launch_bounds__(256) void tindex_count_kernel(const int32_t *__restrict__ idx, int L, HeadTable tab,
                                                           int32_t *__restrict__ cnt)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int32_t *base = idx + tab.off[slot];
    int32_t *c = cnt + (int64_t)bh * L;
    for (int64_t i = blockIdx.x; i < L; i += gridDim.x) {
        const int32_t *row = base + i * k;
        for (int t = threadIdx.x; t < k; t += 256) atomicAdd(&c[row[t]], 1);
    }
}

// One block per (b, h): exclusive scan of cnt into col (int64, L+1 entries); cnt is reset to zero
// so that the fill pass can reuse it as the cursor array.
__global__ __launch_bounds__(1024) void tindex_scan_kernel(int32_t *__restrict__ cnt, int64_t *__restrict__ col, int L)
{
    __shared__ int64_t part[1024];
    const int bh = blockIdx.x;
    int32_t *c = cnt + (int64_t)bh * L;
    int64_t *o = col + (int64_t)bh * (L + 1);
    const int per = (L + 1023) / 1024;
    const int lo = min((int)threadIdx.x * per, L), hi = min(lo + per, L);
    int64_t sum = 0;
    for (int j = lo; j < hi; ++j) sum += c[j];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int step = 1; step < 1024; step <<= 1) {
        int64_t add = threadIdx.x >= (unsigned)step ? part[threadIdx.x - step] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int64_t run = part[threadIdx.x] - sum;
    for (int j = lo; j < hi; ++j) {
        const int32_t v = c[j];
        o[j] = run;
        run += v;
        c[j] = 0;
    }
    if (threadIdx.x == 1023) o[L] = part[1023];
}

__global__ __launch_bounds__(256) void tindex_fill_kernel(const int32_t *__restrict__ idx, int L, HeadTable tab,
                                                          int32_t *__restrict__ cursor,
                                                          const int64_t *__restrict__ col, int32_t *__restrict__ idxT)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int32_t *base = idx + tab.off[slot];
    int32_t *out = idxT + tab.off[slot];
    int32_t *cur = cursor + (int64_t)bh * L;
    const int64_t *cp = col + (int64_t)bh * (L + 1);
    for (int64_t i = blockIdx.x; i < L; i += gridDim.x) {
        const int32_t *row = base + i * k;
        for (int t = threadIdx.x; t < k; t += 256) {
            const int j = row[t];
            const int pos = atomicAdd(&cur[j], 1);
            out[cp[j] + pos] = (int32_t)i;
        }
    }
}

// dkdv pass: a group of 16 lanes owns key j and walks the queries that selected it.
//   dK_j = scale * sum_i dS_ij q_i,  dV_j = sum_i p_ij dO_i,  dS_ij = p_ij (dO_i . v_j - Delta_i).
// Keys with an empty list get zeros; every output row is written exactly once.
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dkdv_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                              const T *__restrict__ V,
                                                              const int32_t *__restrict__ idxT,
                                                              const int64_t *__restrict__ col,
                                                              const float *__restrict__ lse,
                                                              const float *__restrict__ delta,
                                                              const T *__restrict__ dO, T *__restrict__ dK,
                                                              T *__restrict__ dV, int L, float scale, HeadTable tab)
{
    constexpr int CH = D / 16;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t jq = (int64_t)blockIdx.x * 16 + wave * 4 + grp;
    const bool live = jq < L;
    const int64_t j = live ? jq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Qb = Q + head_base + s * CH;
    const T *Gb = dO + head_base + s * CH;
    const float *lse_b = lse + (int64_t)bh * L;
    const float *delta_b = delta + (int64_t)bh * L;
    const int64_t *cp = col + (int64_t)bh * (L + 1);
    const int64_t beg = cp[j];
    const int n = live ? (int)(cp[j + 1] - beg) : 0;
    const int32_t *list = idxT + tab.off[slot] + beg;

    const Chunk kc = load_chunk<T, CH>(K + head_base + j * D + s * CH);
    const Chunk vc = load_chunk<T, CH>(V + head_base + j * D + s * CH);
    const float c2 = scale * kLog2e;

    float dk[CH], dv[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { dk[c] = 0.f; dv[c] = 0.f; }

    // every group of the wave runs the longest list's trip count; shorter lists idle with p = 0
    int nmax = n;
    nmax = max(nmax, __shfl_xor(nmax, 16));
    nmax = max(nmax, __shfl_xor(nmax, 32));
    for (int t0 = 0; t0 < nmax; t0 += U) {
        int iq[U];
        Chunk qc[U], gc[U];
        float l2[U], dl[U];
#pragma unroll
        for (int u = 0; u < U; ++u) iq[u] = (t0 + u < n) ? list[t0 + u] : (int)j;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            qc[u] = load_chunk<T, CH>(Qb + (int64_t)iq[u] * D);
            gc[u] = load_chunk<T, CH>(Gb + (int64_t)iq[u] * D);
            l2[u] = lse_b[iq[u]] * kLog2e;
            dl[u] = delta_b[iq[u]];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float sc = row16_sum(dot_chunk<T, CH>(qc[u], kc));
            const float dp = row16_sum(dot_chunk<T, CH>(gc[u], vc));
            const float p = (t0 + u < n) ? exp2f(sc * c2 - l2[u]) : 0.f;
            const float ds = p * (dp - dl[u]);
            float qf[CH], gf[CH];
            unpack_chunk<T, CH>(qc[u], qf);
            unpack_chunk<T, CH>(gc[u], gf);
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                dk[c] = fmaf(ds, qf[c], dk[c]);
                dv[c] = fmaf(p, gf[c], dv[c]);
            }
        }
    }
    if (live) {
#pragma unroll
        for (int c = 0; c < CH; ++c) dk[c] *= scale;
        store_chunk<T, CH>(dK + head_base + j * D + s * CH, dk);
        store_chunk<T, CH>(dV + head_base + j * D + s * CH, dv);
    }
}

__global__ __launch_bounds__(256) void fill_zero_i32_kernel(int4 *__restrict__ p, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n4; e += stride) p[e] = make_int4(0, 0, 0, 0);
}

// ------------------------------------------------------------------------------------ host
template <typename T, int D>
static dsv_status fwd_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                        const void *V, const int32_t *idx, void *O, float *lse, hipStream_t st)
{
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((p.L + 15) / 16, tabs[t].n);
        hipLaunchKernelGGL((sparse_fwd_kernel<T, D>), grid, dim3(256), 0, st, (const T *)Q, (const T *)K, (const T *)V,
                           idx, (T *)O, lse, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

dsv_status launch_sparse_fwd(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idx, void *O, float *lse, hipStream_t st)
{
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) return fwd_t<bf16_t, 64>(p, tabs, n_tabs, Q, K, V, idx, O, lse, st);
        if (p.d == 128) return fwd_t<bf16_t, 128>(p, tabs, n_tabs, Q, K, V, idx, O, lse, st);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) return fwd_t<float, 64>(p, tabs, n_tabs, Q, K, V, idx, O, lse, st);
        if (p.d == 128) return fwd_t<float, 128>(p, tabs, n_tabs, Q, K, V, idx, O, lse, st);
    }
    return DSV_EUNSUPPORTED;
}

template <typename T, int D>
static dsv_status bwd_dq_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                           const void *V, const int32_t *idx, const float *lse, const void *dO, void *dQ,
                           float *delta, hipStream_t st)
{
    for (int t = 0; t < n_tabs; ++t) {
        dim3 qgrid((p.L + 15) / 16, tabs[t].n);
        hipLaunchKernelGGL((sparse_bwd_dq_kernel<T, D>), qgrid, dim3(256), 0, st, (const T *)Q, (const T *)K,
                           (const T *)V, idx, lse, (const T *)dO, (T *)dQ, delta, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dkdv_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idxT, const int64_t *col, const float *lse,
                             const float *delta, const void *dO, void *dK, void *dV, hipStream_t st)
{
    for (int t = 0; t < n_tabs; ++t) {
        dim3 kgrid((p.L + 15) / 16, tabs[t].n);
        hipLaunchKernelGGL((sparse_bwd_dkdv_kernel<T, D>), kgrid, dim3(256), 0, st, (const T *)Q, (const T *)K,
                           (const T *)V, idxT, col, lse, delta, (const T *)dO, (T *)dK, (T *)dV, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

#define DSV_DISPATCH_TD(FN, ...)                                        \
    do {                                                                \
        if (p.dtype == DSV_BF16) {                                      \
            if (p.d == 64) return FN<bf16_t, 64>(__VA_ARGS__);          \
            if (p.d == 128) return FN<bf16_t, 128>(__VA_ARGS__);        \
        } else if (p.dtype == DSV_F32) {                                \
            if (p.d == 64) return FN<float, 64>(__VA_ARGS__);           \
            if (p.d == 128) return FN<float, 128>(__VA_ARGS__);         \
        }                                                               \
        return DSV_EUNSUPPORTED;                                        \
    } while (0)

dsv_status launch_bwd_dq(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                         const void *V, const int32_t *idx, const float *lse, const void *dO, void *dQ, float *delta,
                         hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dq_t, p, tabs, n_tabs, Q, K, V, idx, lse, dO, dQ, delta, st);
}

dsv_status launch_bwd_dkdv(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                           const void *V, const int32_t *idxT, const int64_t *col, const float *lse, const float *delta,
                           const void *dO, void *dK, void *dV, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dkdv_t, p, tabs, n_tabs, Q, K, V, idxT, col, lse, delta, dO, dK, dV, st);
}

dsv_status launch_idx_transpose(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const int32_t *idx,
                                int32_t *idxT, int64_t *col, int32_t *cnt, size_t cnt_bytes, hipStream_t st)
{
    const int nbh = p.B * p.H;
    const int64_t ncnt4 = (int64_t)(cnt_bytes / 16);
    const int zero_blocks = (int)std::min<int64_t>((ncnt4 + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_i32_kernel, dim3(zero_blocks), dim3(256), 0, st, (int4 *)cnt, ncnt4);
    DSV_LAUNCH_CHECK();
    const int row_blocks = std::min(p.L, 8192);
    for (int t = 0; t < n_tabs; ++t) {
        hipLaunchKernelGGL(tindex_count_kernel, dim3(row_blocks, tabs[t].n), dim3(256), 0, st, idx, p.L, tabs[t], cnt);
        DSV_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(tindex_scan_kernel, dim3(nbh), dim3(1024), 0, st, cnt, col, p.L);
    DSV_LAUNCH_CHECK();
    for (int t = 0; t < n_tabs; ++t) {
        hipLaunchKernelGGL(tindex_fill_kernel, dim3(row_blocks, tabs[t].n), dim3(256), 0, st, idx, p.L, tabs[t], cnt, col,
                           idxT);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

}  // namespace dsv
