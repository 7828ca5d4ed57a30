// Stage 2, order-agnostic form: exact softmax attention over the selected KV only, forward and
// backward (paper Sec. "Sparse Attention with Query Grouping", per-query form; attention formula
// of Sec. "Various Self-Attention Paradigms"), for index rows in ANY order; also the generic
// index transposition.  The inner loops live in stage2_core.h.
//
// A wave handles 4 rows (one per 16-lane group), a block 16 consecutive rows of one head.
#include <algorithm>

#include "stage2_core.h"

namespace dsv {

// ------------------------------------------------------------------------------------ forward
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_fwd_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                         const T *__restrict__ V, const int32_t *__restrict__ idx,
                                                         T *__restrict__ O, float *__restrict__ lse, int L,
                                                         float scale, HeadTable tab)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t iq = (int64_t)blockIdx.x * (4 * RPW) + wave * RPW + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const int32_t *row = idx + tab.off[slot] + i * k;

    const RowChunk<T, CH> q = load_chunk<T, CH, LL::PSB>(Q + head_base + i * D + LL::off(s));
    FwdState<CH> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) st.acc[c] = 0.f;
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];  // one index staging slot per row group
    int32_t *stage = stage_all[threadIdx.x / LPR];
    fwd_sweep<T, D, LPR>(st, q, K + head_base, V + head_base, (uint32_t)LL::off(s), row, 0, k, scale * kLog2e, stage, s);

    const float inv = 1.f / st.l;
#pragma unroll
    for (int c = 0; c < CH; ++c) st.acc[c] *= inv;
    if (live) {
        store_chunk<T, CH, LL::PSB>(O + head_base + i * D + LL::off(s), st.acc);
        if (s == 0) lse[(int64_t)bh * L + i] = (st.m + log2f(st.l)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------ backward
// Two gather passes with no floating-point atomics:
//   dq pass    query-major over idx: dQ and the row term Delta_i;
//   dkdv pass  key-major over the transposed index (for each key, the queries that selected it):
//              dK and dV, each output row owned by one lane group.
// Delta_i = dO_i . O_i equals sum_j p_ij dP_ij over the selected keys (dP_ij = dO_i . v_j); the dq
// pass forms it from that sum in fp32, because the stored O is rounded to the storage type and the
// error of dO . O_stored alone would exceed the output tolerance.  One sweep yields both Delta and dQ:
// with D0 = dO_i . O_stored as a centring value,
//   dQ_i = scale * ( sum_j p_ij (dP_ij - D0) k_j  -  (Delta_i - D0) * sum_j p_ij k_j ).
// Delta is kept for the dkdv pass.
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_bwd_dq_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                            const T *__restrict__ V,
                                                            const int32_t *__restrict__ idx, const T *__restrict__ O,
                                                            const float *__restrict__ lse, const T *__restrict__ dO,
                                                            T *__restrict__ dQ, float *__restrict__ delta_out, int L,
                                                            float scale, HeadTable tab)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t iq = (int64_t)blockIdx.x * (4 * RPW) + wave * RPW + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const int32_t *row = idx + tab.off[slot] + i * k;

    const RowChunk<T, CH> q = load_chunk<T, CH, LL::PSB>(Q + head_base + i * D + LL::off(s));
    const RowChunk<T, CH> go = load_chunk<T, CH, LL::PSB>(dO + head_base + i * D + LL::off(s));
    const RowChunk<T, CH> o = load_chunk<T, CH, LL::PSB>(O + head_base + i * D + LL::off(s));
    const float delta0 = row_sum<LPR>(dot_chunk<T, CH>(go, o));
    DqState<CH> st;
    st.delta = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) { st.a[c] = 0.f; st.b[c] = 0.f; }
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];  // one index staging slot per row group
    int32_t *stage = stage_all[threadIdx.x / LPR];
    dq_sweep<T, D, LPR>(st, q, go, K + head_base, V + head_base, (uint32_t)LL::off(s), row, 0, k, scale * kLog2e,
                   lse[(int64_t)bh * L + i] * kLog2e, delta0, stage, s);
    if (live) {
        float dq[CH];
#pragma unroll
        for (int c = 0; c < CH; ++c) dq[c] = scale * (st.a[c] - (st.delta - delta0) * st.b[c]);
        store_chunk<T, CH, LL::PSB>(dQ + head_base + i * D + LL::off(s), dq);
        if (s == 0) delta_out[(int64_t)bh * L + i] = st.delta;
    }
}

// dkdv pass: a group of 16 lanes owns key j and walks the queries that selected it.
//   dK_j = scale * sum_i dS_ij q_i,  dV_j = sum_i p_ij dO_i,  dS_ij = p_ij (dO_i . v_j - Delta_i).
// Keys with an empty list get zeros; every output row is written exactly once.
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_bwd_dkdv_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                              const T *__restrict__ V,
                                                              const int32_t *__restrict__ idxT,
                                                              const int64_t *__restrict__ col,
                                                              const float *__restrict__ lse,
                                                              const float *__restrict__ delta,
                                                              const T *__restrict__ dO, T *__restrict__ dK,
                                                              T *__restrict__ dV, int L, float scale, HeadTable tab)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t jq = (int64_t)blockIdx.x * (4 * RPW) + wave * RPW + grp;
    const bool live = jq < L;
    const int64_t j = live ? jq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const int64_t *cp = col + (int64_t)bh * (L + 1);
    const int64_t beg = cp[j];
    const int n = live ? (int)(cp[j + 1] - beg) : 0;
    const int32_t *list = idxT + tab.off[slot] + beg;

    const RowChunk<T, CH> kc = load_chunk<T, CH, LL::PSB>(K + head_base + j * D + LL::off(s));
    const RowChunk<T, CH> vc = load_chunk<T, CH, LL::PSB>(V + head_base + j * D + LL::off(s));
    DkdvState<CH> st;
#pragma unroll
    for (int c = 0; c < CH; ++c) { st.dk[c] = 0.f; st.dv[c] = 0.f; }
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];  // one index staging slot per row group
    int32_t *stage = stage_all[threadIdx.x / LPR];
    dkdv_sweep<T, D, LPR>(st, kc, vc, Q + head_base, dO + head_base, lse + (int64_t)bh * L, delta + (int64_t)bh * L,
                     (uint32_t)LL::off(s), list, 0, n, scale * kLog2e, stage, s);
    if (live) {
#pragma unroll
        for (int c = 0; c < CH; ++c) st.dk[c] *= scale;
        store_chunk<T, CH, LL::PSB>(dK + head_base + j * D + LL::off(s), st.dk);
        store_chunk<T, CH, LL::PSB>(dV + head_base + j * D + LL::off(s), st.dv);
    }
}

// ---- transposed index: for every key, the list of queries whose row holds it ----------------
// A stable counting sort by key, so that every list comes out in ascending query order whatever the order inside the
// rows is (the L2-blocked key-major sweep needs ascending lists) and the result is the same from run to run:
//   count    the queries are cut into chunks of consecutive rows; cnt2[bh, chunk, j] = rows of the chunk holding j
//            (integer atomics: the counts do not depend on the order of arrival);
//   offsets  per key, an exclusive scan over the chunks (cnt2 becomes the chunk's first position inside the key's
//            list) and the key's total; the totals are scanned into col as before;
//   fill     one block per chunk walks its rows in ascending order, one row at a time; the entries of a row are
//            distinct keys, so the threads bump the chunk's cursors with plain loads and stores.
constexpr int kTransposeChunks = 256;  // at most this many query chunks per head (cnt2 holds chunks x L counters; 1024
                                       // chunks measured no faster: both passes are bound by scattered 4-byte requests)

__host__ __device__ __forceinline__ int transpose_chunk_rows(int L)
{
    const int r = (L + kTransposeChunks - 1) / kTransposeChunks;
    return r < 64 ? 64 : r;
}

__global__ __launch_bounds__(256) void tindex_count_kernel(const int32_t *__restrict__ idx, int L, int n_chunks,
                                                           HeadTable tab, int32_t *__restrict__ cnt2)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int rc = transpose_chunk_rows(L);
    const int chunk = blockIdx.x;
    const int32_t *base = idx + tab.off[slot];
    int32_t *c = cnt2 + ((int64_t)bh * n_chunks + chunk) * L;
    const int i1 = min((chunk + 1) * rc, L);
    for (int64_t i = (int64_t)chunk * rc; i < i1; ++i) {
        const int32_t *row = base + i * k;
        for (int t = threadIdx.x; t < k; t += 256) {
            const int j = row[t];
            if (j >= 0 && j < L) atomicAdd(&c[j], 1);
        }
    }
}

// thread per key: cnt2[bh, c, j] <- number of rows in chunks before c holding j; tot[bh, j] <- all of them
__global__ __launch_bounds__(256) void tindex_offsets_kernel(int32_t *__restrict__ cnt2, int32_t *__restrict__ tot, int L,
                                                             int n_chunks)
{
    const int bh = blockIdx.y;
    const int j = blockIdx.x * 256 + threadIdx.x;
    if (j >= L) return;
    int32_t *c = cnt2 + (int64_t)bh * n_chunks * L + j;
    int run = 0;
    for (int ch = 0; ch < n_chunks; ++ch) {
        const int v = c[(int64_t)ch * L];
        c[(int64_t)ch * L] = run;
        run += v;
    }
    tot[(int64_t)bh * L + j] = run;
}

// One block per (b, h): exclusive scan of cnt into col (int64, L+1 entries).
__global__ __launch_bounds__(1024) void tindex_scan_kernel(const int32_t *__restrict__ cnt, int64_t *__restrict__ col, int L)
{
    __shared__ int64_t part[1024];
    const int bh = blockIdx.x;
    const int32_t *c = cnt + (int64_t)bh * L;
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
        o[j] = run;
        run += c[j];
    }
    if (threadIdx.x == 1023) o[L] = part[1023];
}

__global__ __launch_bounds__(256) void tindex_fill_kernel(const int32_t *__restrict__ idx, int L, int n_chunks,
                                                          HeadTable tab, int32_t *__restrict__ cnt2,
                                                          const int64_t *__restrict__ col, int32_t *__restrict__ idxT)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int rc = transpose_chunk_rows(L);
    const int chunk = blockIdx.x;
    const int32_t *base = idx + tab.off[slot];
    int32_t *out = idxT + tab.off[slot];
    int32_t *cur = cnt2 + ((int64_t)bh * n_chunks + chunk) * L;  // this chunk's next position inside every list
    const int64_t *cp = col + (int64_t)bh * (L + 1);
    const int i1 = min((chunk + 1) * rc, L);
    constexpr int U = 8;  // entries a thread has in flight: the loads of all U come before the first store
    for (int64_t i = (int64_t)chunk * rc; i < i1; ++i) {
        const int32_t *row = base + i * k;
        for (int t0 = threadIdx.x; t0 < k; t0 += 256 * U) {
            int j[U], pos[U];
            int64_t dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0 + u * 256;
                j[u] = t < k ? row[t] : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const bool ok = j[u] >= 0 && j[u] < L;
                pos[u] = ok ? cur[j[u]] : 0;   // no other thread touches cur[j] during this row: a row's keys are distinct
                dst[u] = ok ? cp[j[u]] + pos[u] : -1;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (j[u] >= 0 && j[u] < L) {
                    cur[j[u]] = pos[u] + 1;
                    // col and the cursors come from the counting pass over the same idx, so dst stays inside the
                    // head's L * k entries; the bound keeps a broken idx (duplicates, changed between the passes)
                    // from sending the store anywhere else
                    if (dst[u] >= 0 && dst[u] < (int64_t)L * k) out[dst[u]] = (int32_t)i;
                }
            }
        }
        __syncthreads();  // the next row may bump the same cursors
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
    KernelSpan span(DSV_KERNEL_FWD_SWEEP, st);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((p.L + 256 / SweepLanes<T, D>::fwd - 1) / (256 / SweepLanes<T, D>::fwd), tabs[t].n);
        hipLaunchKernelGGL((sparse_fwd_kernel<T, D, SweepLanes<T, D>::fwd>), grid, dim3(256), 0, st, (const T *)Q, (const T *)K, (const T *)V,
                           idx, (T *)O, lse, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dq_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                           const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO,
                           void *dQ, float *delta, hipStream_t st)
{
    KernelSpan span(DSV_KERNEL_DQ_SWEEP, st);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 qgrid((p.L + 256 / SweepLanes<T, D>::dq - 1) / (256 / SweepLanes<T, D>::dq), tabs[t].n);
        hipLaunchKernelGGL((sparse_bwd_dq_kernel<T, D, SweepLanes<T, D>::dq>), qgrid, dim3(256), 0, st, (const T *)Q, (const T *)K,
                           (const T *)V, idx, (const T *)O, lse, (const T *)dO, (T *)dQ, delta, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dkdv_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idxT, const int64_t *col, const float *lse,
                             const float *delta, const void *dO, void *dK, void *dV, hipStream_t st)
{
    KernelSpan span(DSV_KERNEL_DKDV_SWEEP, st);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 kgrid((p.L + 256 / SweepLanes<T, D>::dkdv - 1) / (256 / SweepLanes<T, D>::dkdv), tabs[t].n);
        hipLaunchKernelGGL((sparse_bwd_dkdv_kernel<T, D, SweepLanes<T, D>::dkdv>), kgrid, dim3(256), 0, st, (const T *)Q, (const T *)K,
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

dsv_status launch_sparse_fwd(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idx, void *O, float *lse, hipStream_t st)
{
    DSV_DISPATCH_TD(fwd_t, p, tabs, n_tabs, Q, K, V, idx, O, lse, st);
}

dsv_status launch_bwd_dq(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                         const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO, void *dQ,
                         float *delta, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dq_t, p, tabs, n_tabs, Q, K, V, idx, O, lse, dO, dQ, delta, st);
}

dsv_status launch_bwd_dkdv(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                           const void *V, const int32_t *idxT, const int64_t *col, const float *lse, const float *delta,
                           const void *dO, void *dK, void *dV, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dkdv_t, p, tabs, n_tabs, Q, K, V, idxT, col, lse, delta, dO, dK, dV, st);
}

size_t idx_transpose_bytes(const dsv_problem &p)
{
    const size_t nbh = (size_t)p.B * p.H;
    const int rc = transpose_chunk_rows(p.L);
    const size_t n_chunks = (size_t)(p.L + rc - 1) / rc;
    return align_up(nbh * p.L * 4, 256) + align_up(nbh * n_chunks * p.L * 4, 256);   // tot, cnt2
}

dsv_status launch_idx_transpose(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const int32_t *idx,
                                int32_t *idxT, int64_t *col, int32_t *cnt, size_t cnt_bytes, hipStream_t st)
{
    const int nbh = p.B * p.H;
    if (cnt_bytes < idx_transpose_bytes(p)) return DSV_EWORKSPACE;
    const int rc = transpose_chunk_rows(p.L);
    const int n_chunks = (p.L + rc - 1) / rc;
    int32_t *tot = cnt;
    int32_t *cnt2 = cnt + align_up((size_t)nbh * p.L * 4, 256) / 4;
    const int64_t ncnt4 = (int64_t)(idx_transpose_bytes(p) / 16);
    const int zero_blocks = (int)std::min<int64_t>((ncnt4 + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_zero_i32_kernel, dim3(zero_blocks), dim3(256), 0, st, (int4 *)cnt, ncnt4);
    DSV_LAUNCH_CHECK();
    for (int t = 0; t < n_tabs; ++t) {
        hipLaunchKernelGGL(tindex_count_kernel, dim3(n_chunks, tabs[t].n), dim3(256), 0, st, idx, p.L, n_chunks, tabs[t], cnt2);
        DSV_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL(tindex_offsets_kernel, dim3((p.L + 255) / 256, nbh), dim3(256), 0, st, cnt2, tot, p.L, n_chunks);
    hipLaunchKernelGGL(tindex_scan_kernel, dim3(nbh), dim3(1024), 0, st, tot, col, p.L);
    DSV_LAUNCH_CHECK();
    for (int t = 0; t < n_tabs; ++t) {
        hipLaunchKernelGGL(tindex_fill_kernel, dim3(n_chunks, tabs[t].n), dim3(256), 0, st, idx, p.L, n_chunks, tabs[t], cnt2,
                           col, idxT);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

}  // namespace dsv
