// Stage 2, L2-blocked form, for index rows (and key-major lists) in ascending order.
//
// The plain gather kernels (stage2.hip) fetch every selected K/V row from wherever it lives; at
// L = 128k a head's K+V slab is 67 MB, far beyond the 4 MB L2 of an XCD, so the gathers are served
// by the memory-side cache at about its bandwidth.  Here the key axis is cut into ranges whose K+V
// rows fit one XCD's L2 with room to spare.  Because a row of idx is ascending, the keys a query
// selected inside one range are one contiguous segment of its row.  Work item = (head, range,
// block of 16 queries); the 1-D grid is laid out so that workgroup b runs on XCD b % 8 and every
// XCD walks "its" ranges one after the other with all of its CUs inside the same range, which
// keeps that range's rows resident in that XCD's L2.  Each item leaves a partial result per row
// (split-K); a small second kernel merges the partials.  The backward's dkdv step does the same
// key-major: lists of queries cut by QUERY ranges, Q / dO rows resident.
//
// Inner loops and lane layout: stage2_core.h.
#include <algorithm>

#include "stage2_core.h"

namespace dsv {

// Decode a linear block id into (head slot, range, row block).  Consecutive ids go to
// consecutive XCDs; ids b, b+8, b+16, ... (one XCD) walk the row blocks of one range, then the
// next range of that XCD.  Ranges are padded to a multiple of 8; padded ranges return false.
__device__ __forceinline__ bool decode_item(const SplitPlan &pl, int64_t b, int &slot, int &range, int &rb)
{
    const int64_t per_head = (int64_t)pl.S_pad * pl.nqb;
    slot = (int)(b / per_head);
    const int64_t rem = b - (int64_t)slot * per_head;
    const int xcd = (int)(rem & 7);
    const int64_t local = rem >> 3;
    const int t = (int)(local / pl.nqb);
    rb = (int)(local - (int64_t)t * pl.nqb);
    range = t * 8 + xcd;
    return range < pl.S;
}

// ---- segment pointers -----------------------------------------------------------------------
// seg[bh, row, s] = first position in the (ascending) row whose value is >= s * range_len, for
// s = 0 .. S.  Query-major: rows of idx (length k).  Key-major: lists of idx_t (start and length
// from col_ptr), cut by QUERY ranges.
__global__ __launch_bounds__(256) void segment_ptr_kernel(const int32_t *__restrict__ index,
                                                          const int64_t *__restrict__ col, int L, HeadTable tab,
                                                          SplitPlan pl, int32_t *__restrict__ seg, GroupExpand ge)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int np = pl.S + 1;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)L * np) return;
    const int row = (int)(e / np);
    const int s = (int)(e - (int64_t)row * np);
    const int32_t *base;
    int len;
    if (col) {
        const int64_t *cp = col + (int64_t)bh * (L + 1);
        base = index + tab.off[slot] + cp[row];
        len = (int)(cp[row + 1] - cp[row]) * ge.G;  // lists of groups: positions of the expanded list
    } else {
        len = tab.k[slot];
        base = index + tab.off[slot] + (int64_t)row * len;
    }
    const int64_t target = (int64_t)s * pl.range_len;
    int lo = 0, hi = len;  // first position with value >= target
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)expanded_entry(base, mid, ge) < target) lo = mid + 1; else hi = mid;
    }
    seg[((int64_t)bh * L + row) * np + s] = lo;
}

// ---- forward ----------------------------------------------------------------------------------
// Partial softmax state of one (query, range): running max m (log2 domain), l = sum 2^(s-m),
// acc = sum 2^(s-m) v.  Empty segments leave (m = -inf, l = 0, acc = 0).
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_fwd_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                               const T *__restrict__ V,
                                                               const int32_t *__restrict__ idx,
                                                               const int32_t *__restrict__ seg,
                                                               const int32_t *__restrict__ order, float *__restrict__ pm,
                                                               float *__restrict__ pl_, float *__restrict__ pacc, int L,
                                                               float scale, HeadTable tab, SplitPlan pl)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    int slot, range, qb;
    if (!decode_item(pl, blockIdx.x, slot, range, qb)) return;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t ipos = (int64_t)qb * (4 * RPW) + wave * RPW + grp;  // position in this range's row order
    const bool live = ipos < L;
    const int64_t i = order[((int64_t)bh * pl.S + range) * L + (live ? ipos : L - 1)];
    const int64_t head_base = (int64_t)bh * L * D;
    const int32_t *row = idx + tab.off[slot] + i * k;
    const int32_t *sp = seg + ((int64_t)bh * L + i) * (pl.S + 1) + range;
    const int tb = sp[0], te = live ? sp[1] : sp[0];

    const RowChunk<T, CH> q = load_chunk<T, CH, LL::PSB>(Q + head_base + i * D + LL::off(s));
    FwdState<CH> st;
    st.m = -INFINITY;
    st.l = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) st.acc[c] = 0.f;
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];  // one index staging slot per row group
    int32_t *stage = stage_all[threadIdx.x / LPR];
    fwd_sweep<T, D, LPR>(st, q, K + head_base, V + head_base, (uint32_t)LL::off(s), row, tb, te, scale * kLog2e, stage, s);
    if (live) {
        const int64_t slot_id = ((int64_t)bh * L + i) * pl.S + range;
        store_acc<T, D, LPR>(pacc + slot_id * D, s, st.acc);
        if (s == 0) { pm[slot_id] = st.m; pl_[slot_id] = st.l; }
    }
}

// Merge the S partial states of every query: O = sum_s w_s acc_s / sum_s w_s l_s, w_s = 2^(m_s - M).
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_fwd_merge_kernel(const float *__restrict__ pm, const float *__restrict__ pl_,
                                                               const float *__restrict__ pacc, T *__restrict__ O,
                                                               float *__restrict__ lse, int64_t n_rows, int S)
{
    constexpr int CH = D / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t row = (int64_t)blockIdx.x * 16 + wave * 4 + grp;  // b*H*L + i
    if (row >= n_rows) return;
    const float *m_r = pm + row * S;
    const float *l_r = pl_ + row * S;
    float M = -INFINITY;
    for (int t = 0; t < S; ++t) M = fmaxf(M, m_r[t]);
    float lsum = 0.f;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;
    for (int t = 0; t < S; ++t) {
        const float w = exp2f(m_r[t] - M);
        lsum = fmaf(w, l_r[t], lsum);
        const RowChunk<float, CH> a = load_chunk<float, CH>(pacc + (row * S + t) * D + s * CH);
#pragma unroll
        for (int c = 0; c < CH; ++c) acc[c] = fmaf(w, __uint_as_float(a.w[c]), acc[c]);
    }
    const float inv = 1.f / lsum;
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] *= inv;
    store_chunk<T, CH>(O + row * D + s * CH, acc);
    if (s == 0) lse[row] = (M + log2f(lsum)) * kLn2;
}

// ---- backward, dq step ---------------------------------------------------------------------------
// Per (query, key range): C = sum p (dP - D0) k, B = sum p k, Delta = sum p dP over the segment, with
// D0 = dO . O_stored (all three are plain sums over the selected keys, so partials simply add).
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_bwd_dq_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                  const T *__restrict__ V,
                                                                  const int32_t *__restrict__ idx,
                                                                  const int32_t *__restrict__ seg,
                                                                  const int32_t *__restrict__ order,
                                                                  const T *__restrict__ O,
                                                                  const float *__restrict__ lse,
                                                                  const T *__restrict__ dO, float *__restrict__ pa,
                                                                  float *__restrict__ pb, float *__restrict__ pdelta,
                                                                  int L, float scale, HeadTable tab, SplitPlan pl)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    int slot, range, qb;
    if (!decode_item(pl, blockIdx.x, slot, range, qb)) return;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t ipos = (int64_t)qb * (4 * RPW) + wave * RPW + grp;  // position in this range's row order
    const bool live = ipos < L;
    const int64_t i = order[((int64_t)bh * pl.S + range) * L + (live ? ipos : L - 1)];
    const int64_t head_base = (int64_t)bh * L * D;
    const int32_t *row = idx + tab.off[slot] + i * k;
    const int32_t *sp = seg + ((int64_t)bh * L + i) * (pl.S + 1) + range;
    const int tb = sp[0], te = live ? sp[1] : sp[0];

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
    dq_sweep<T, D, LPR>(st, q, go, K + head_base, V + head_base, (uint32_t)LL::off(s), row, tb, te, scale * kLog2e,
                   lse[(int64_t)bh * L + i] * kLog2e, delta0, stage, s);
    if (live) {
        const int64_t slot_id = ((int64_t)bh * L + i) * pl.S + range;
        store_acc<T, D, LPR>(pa + slot_id * D, s, st.a);
        store_acc<T, D, LPR>(pb + slot_id * D, s, st.b);
        if (s == 0) pdelta[slot_id] = st.delta;
    }
}

// dQ_i = scale * (sum_s C_s - (Delta_i - D0) * sum_s B_s), Delta_i = sum_s Delta_s, D0 = dO_i . O_i(stored).
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dq_merge_kernel(const float *__restrict__ pa,
                                                                  const float *__restrict__ pb,
                                                                  const float *__restrict__ pdelta,
                                                                  const T *__restrict__ O, const T *__restrict__ dO,
                                                                  T *__restrict__ dQ, float *__restrict__ delta_out,
                                                                  int64_t n_rows, int S, float scale)
{
    constexpr int CH = D / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t row = (int64_t)blockIdx.x * 16 + wave * 4 + grp;
    if (row >= n_rows) return;
    float a[CH], b[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { a[c] = 0.f; b[c] = 0.f; }
    float delta = 0.f;
    for (int t = 0; t < S; ++t) {
        const RowChunk<float, CH> ca = load_chunk<float, CH>(pa + (row * S + t) * D + s * CH);
        const RowChunk<float, CH> cb = load_chunk<float, CH>(pb + (row * S + t) * D + s * CH);
        delta += pdelta[row * S + t];
#pragma unroll
        for (int c = 0; c < CH; ++c) { a[c] += __uint_as_float(ca.w[c]); b[c] += __uint_as_float(cb.w[c]); }
    }
    const RowChunk<T, CH> go = load_chunk<T, CH>(dO + row * D + s * CH);
    const RowChunk<T, CH> o = load_chunk<T, CH>(O + row * D + s * CH);
    const float delta0 = row16_sum(dot_chunk<T, CH>(go, o));  // the sweep reduced the same products over another lane layout: equal up to fp32 rounding (~1e-6), far below what the centring needs
    float dq[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) dq[c] = scale * (a[c] - (delta - delta0) * b[c]);
    store_chunk<T, CH>(dQ + row * D + s * CH, dq);
    if (s == 0) delta_out[row] = delta;
}

// ---- backward, dkdv step -------------------------------------------------------------------------
// Key-major: work item = (head, QUERY range, block of 16 keys); a key's ascending query list has one
// contiguous segment per query range, whose Q / dO rows (and lse, Delta entries) stay in L2.
// `order`: this range's keys by descending segment length (see seglen_* below).
// The block first parks the range's {lse * log2(e), Delta} entries (8 bytes per query, dynamic LDS of range_len
// entries: at most 64 KB, two blocks per CU, which is what the registers allow anyway) and the sweep reads them
// from there: one vector-memory access less per pair.
template <typename T, int D, int LPR>
__global__ __launch_bounds__(256) void sparse_bwd_dkdv_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                    const T *__restrict__ V,
                                                                    const int32_t *__restrict__ idxT,
                                                                    const int64_t *__restrict__ col,
                                                                    const int32_t *__restrict__ seg,
                                                                    const int32_t *__restrict__ order,
                                                                    const float2 *__restrict__ rowstat,
                                                                    const T *__restrict__ dO, float *__restrict__ pdk,
                                                                    float *__restrict__ pdv, int L, float scale,
                                                                    HeadTable tab, SplitPlan pl, GroupExpand ge)
{
    typedef LaneLayout<T, D, LPR> LL;
    constexpr int CH = D / LPR;
    constexpr int RPW = 64 / LPR;  // rows per wave
    int slot, range, kb;
    if (!decode_item(pl, blockIdx.x, slot, range, kb)) return;
    const int bh = tab.bh[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane / LPR, s = lane % LPR;
    const int64_t jpos = (int64_t)kb * (4 * RPW) + wave * RPW + grp;
    const bool live = jpos < L;
    const int64_t jp = live ? jpos : L - 1;
    const int64_t j = order[((int64_t)bh * pl.S + range) * L + jp];
    const int64_t head_base = (int64_t)bh * L * D;
    const int32_t *list = idxT + tab.off[slot] + col[(int64_t)bh * (L + 1) + j];
    const int32_t *sp = seg + ((int64_t)bh * L + j) * (pl.S + 1) + range;
    const int tb = sp[0], te = live ? sp[1] : sp[0];

    const RowChunk<T, CH> kc = load_chunk<T, CH, LL::PSB>(K + head_base + j * D + LL::off(s));
    const RowChunk<T, CH> vc = load_chunk<T, CH, LL::PSB>(V + head_base + j * D + LL::off(s));
    DkdvState<CH> st;
#pragma unroll
    for (int c = 0; c < CH; ++c) { st.dk[c] = 0.f; st.dv[c] = 0.f; }
    __shared__ __align__(16) int32_t stage_all[256 / LPR][kStage];  // one index staging slot per row group
    int32_t *stage = stage_all[threadIdx.x / LPR];
    extern __shared__ __align__(16) float2 stat_s[];  // [range_len]
    const int q_first = range * pl.range_len;          // first query of this range
    {
        const float2 *src = rowstat + (int64_t)bh * L + q_first;
        const int nq = min(pl.range_len, L - q_first);
        for (int e = threadIdx.x; e < nq; e += 256) stat_s[e] = src[e];
        __syncthreads();
    }
    dkdv_sweep<T, D, LPR, true>(st, kc, vc, Q + head_base, dO + head_base, nullptr, nullptr, (uint32_t)LL::off(s), list, tb,
                                te, scale * kLog2e, stage, s, stat_s, q_first, ge);
    if (live) {
        const int64_t slot_id = ((int64_t)bh * L + j) * pl.S + range;
        store_acc<T, D, LPR>(pdk + slot_id * D, s, st.dk);
        store_acc<T, D, LPR>(pdv + slot_id * D, s, st.dv);
    }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dkdv_merge_kernel(const float *__restrict__ pdk,
                                                                    const float *__restrict__ pdv,
                                                                    T *__restrict__ dK, T *__restrict__ dV,
                                                                    int64_t n_rows, int S, float scale)
{
    constexpr int CH = D / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t row = (int64_t)blockIdx.x * 16 + wave * 4 + grp;
    if (row >= n_rows) return;
    float a[CH], b[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { a[c] = 0.f; b[c] = 0.f; }
    for (int t = 0; t < S; ++t) {
        const RowChunk<float, CH> ca = load_chunk<float, CH>(pdk + (row * S + t) * D + s * CH);
        const RowChunk<float, CH> cb = load_chunk<float, CH>(pdv + (row * S + t) * D + s * CH);
#pragma unroll
        for (int c = 0; c < CH; ++c) { a[c] += __uint_as_float(ca.w[c]); b[c] += __uint_as_float(cb.w[c]); }
    }
#pragma unroll
    for (int c = 0; c < CH; ++c) a[c] *= scale;
    store_chunk<T, CH>(dK + row * D + s * CH, a);
    store_chunk<T, CH>(dV + row * D + s * CH, b);
}

// {lse * log2(e), Delta} of every query side by side, so that the dkdv sweep fetches both with one load.
__global__ __launch_bounds__(256) void pack_rowstat_kernel(const float *__restrict__ lse, const float *__restrict__ delta,
                                                           float2 *__restrict__ out, int64_t n)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) out[e] = make_float2(lse[e] * kLog2e, delta[e]);
}

// ---- row order per range ---------------------------------------------------------------------
// The rows a wave works on together should have segments of the same length in the range at hand,
// or its lanes idle until the longest one is done (uniformly random selections: 7-8 % of the sweep).
// So every (head, range) gets its own order of the L rows, by descending segment length: a counting
// sort on the length (at most range_len).  hist: [B*H, S, nbins] counters, nbins <= range_len + 1;
// order: [B*H, S, L].  The order inside a length class comes from atomic cursors and may differ from
// run to run; results do not depend on it (rows are independent).
// Rows are handled kSeglenChunk at a time by one block per (head, range, chunk), which first counts
// in LDS and then touches the global counters once per length class it has seen (the lengths of a
// range cluster on ~100 values, so per-row global atomics would all hit the same few addresses).
constexpr int kSeglenChunk = 4096;

__device__ __forceinline__ int seg_len(const int32_t *__restrict__ seg, int64_t bh, int L, int S, int row, int r, int nbins)
{
    const int32_t *sp = seg + (bh * L + row) * (S + 1) + r;
    return max(0, min(sp[1] - sp[0], nbins - 1));  // clamped both ways: the result indexes LDS counters
}

__global__ __launch_bounds__(256) void seglen_hist_kernel(const int32_t *__restrict__ seg, int L, int S, int nbins,
                                                          int32_t *__restrict__ hist)
{
    extern __shared__ int32_t lh[];  // [nbins]
    const int nchunks = (L + kSeglenChunk - 1) / kSeglenChunk;
    const int unit = blockIdx.x / nchunks;  // (head, range)
    const int bh = unit / S, r = unit % S;
    const int row0 = (blockIdx.x % nchunks) * kSeglenChunk;
    for (int e = threadIdx.x; e < nbins; e += 256) lh[e] = 0;
    __syncthreads();
    for (int row = row0 + threadIdx.x; row < min(row0 + kSeglenChunk, L); row += 256)
        atomicAdd(&lh[nbins - 1 - seg_len(seg, bh, L, S, row, r, nbins)], 1);
    __syncthreads();
    int32_t *gh = hist + ((int64_t)bh * S + r) * nbins;
    for (int e = threadIdx.x; e < nbins; e += 256)
        if (lh[e]) atomicAdd(&gh[e], lh[e]);
}

// exclusive scan of every [n]-segment of hist (one block per segment)
__global__ __launch_bounds__(1024) void seglen_scan_kernel(int32_t *__restrict__ hist, int n)
{
    __shared__ int32_t part[1024];
    int32_t *h = hist + (int64_t)blockIdx.x * n;
    const int per = (n + 1023) / 1024;
    const int lo = min((int)threadIdx.x * per, n), hi = min(lo + per, n);
    int32_t sum = 0;
    for (int e = lo; e < hi; ++e) sum += h[e];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int step = 1; step < 1024; step <<= 1) {
        const int32_t add = threadIdx.x >= (unsigned)step ? part[threadIdx.x - step] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int32_t run = part[threadIdx.x] - sum;
    for (int e = lo; e < hi; ++e) {
        const int32_t v = h[e];
        h[e] = run;
        run += v;
    }
}

__global__ __launch_bounds__(256) void seglen_scatter_kernel(const int32_t *__restrict__ seg, int L, int S, int nbins,
                                                             int32_t *__restrict__ hist, int32_t *__restrict__ order)
{
    extern __shared__ int32_t lh[];  // [nbins]: this chunk's count per class, then its next free slot in `order`
    const int nchunks = (L + kSeglenChunk - 1) / kSeglenChunk;
    const int unit = blockIdx.x / nchunks;  // (head, range)
    const int bh = unit / S, r = unit % S;
    const int row0 = (blockIdx.x % nchunks) * kSeglenChunk, row1 = min(row0 + kSeglenChunk, L);
    for (int e = threadIdx.x; e < nbins; e += 256) lh[e] = 0;
    __syncthreads();
    for (int row = row0 + threadIdx.x; row < row1; row += 256)
        atomicAdd(&lh[nbins - 1 - seg_len(seg, bh, L, S, row, r, nbins)], 1);
    __syncthreads();
    int32_t *gh = hist + ((int64_t)bh * S + r) * nbins;
    for (int e = threadIdx.x; e < nbins; e += 256)
        if (lh[e]) lh[e] = atomicAdd(&gh[e], lh[e]);  // reserve this chunk's slots of the class
    __syncthreads();
    int32_t *out = order + ((int64_t)bh * S + r) * L;
    for (int row = row0 + threadIdx.x; row < row1; row += 256) {
        // slots come from the counting pass over the same seg, so they stay below L; the bound keeps an
        // inconsistent seg from sending the store out of this (head, range)'s L entries
        const int slot = atomicAdd(&lh[nbins - 1 - seg_len(seg, bh, L, S, row, r, nbins)], 1);
        if (slot >= 0 && slot < L) out[slot] = row;
    }
}

__global__ __launch_bounds__(256) void zero_i32_kernel(int32_t *__restrict__ p, int64_t n)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n; e += stride) p[e] = 0;
}

// ------------------------------------------------------------------------------------ host
SplitPlan make_split_plan(const dsv_problem &p, size_t range_bytes)
{
    const size_t esz = p.dtype == DSV_BF16 ? 2 : 4;
    const size_t row_pair_bytes = 2 * (size_t)p.d * esz;  // one K row + one V row (or Q + dO)
    SplitPlan pl;
    // ranges of about range_bytes, their number a multiple of 8 so that every XCD gets the same
    // number of ranges (a 6-5 split of ranges over XCDs costs ~10 %)
    // at most kMaxRangeRows rows per range: the dkdv sweep parks the range's row statistics in LDS
    const size_t target = std::min<size_t>(kMaxRangeRows, std::max<size_t>(256, range_bytes / row_pair_bytes));
    int S = (int)((p.L + 8 * target - 1) / (8 * target)) * 8;
    pl.range_len = (p.L + S - 1) / S;
    pl.S = (p.L + pl.range_len - 1) / pl.range_len;
    pl.S_pad = (pl.S + 7) / 8 * 8;
    pl.nqb = (p.L + 15) / 16;
    return pl;
}

static dsv_status launch_segments(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const SplitPlan &pl,
                                  const int32_t *index, const int64_t *col, int32_t *seg, hipStream_t st,
                                  GroupExpand ge = no_expand())
{
    const int64_t n = (int64_t)p.L * (pl.S + 1);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((unsigned)((n + 255) / 256), tabs[t].n);
        hipLaunchKernelGGL(segment_ptr_kernel, grid, dim3(256), 0, st, index, col, p.L, tabs[t], pl, seg, ge);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

// order[bh, r, :] = the rows of head bh by descending segment length in range r (from seg).
static dsv_status launch_row_order(const dsv_problem &p, const SplitPlan &pl, const int32_t *seg, int32_t *hist,
                                   int32_t *order, hipStream_t st)
{
    const int nbh = p.B * p.H;
    // length classes; longer segments (possible only with ranges above 8192 rows) share the last class
    const int nbins = std::min(pl.range_len + 1, 8193);
    const int64_t nh = (int64_t)nbh * pl.S * nbins;
    hipLaunchKernelGGL(zero_i32_kernel, dim3((unsigned)std::min<int64_t>((nh + 255) / 256, 4096)), dim3(256), 0, st, hist, nh);
    const int64_t nblocks = (int64_t)((p.L + kSeglenChunk - 1) / kSeglenChunk) * nbh * pl.S;
    if (nblocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
    dim3 grid((unsigned)nblocks);
    hipLaunchKernelGGL(seglen_hist_kernel, grid, dim3(256), (size_t)nbins * 4, st, seg, p.L, pl.S, nbins, hist);
    hipLaunchKernelGGL(seglen_scan_kernel, dim3(nbh * pl.S), dim3(1024), 0, st, hist, nbins);
    hipLaunchKernelGGL(seglen_scatter_kernel, grid, dim3(256), (size_t)nbins * 4, st, seg, p.L, pl.S, nbins, hist, order);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status fwd_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                              const void *V, const int32_t *idx, void *O, float *lse, const SplitPlan &pl,
                              const FwdSplitWorkspace &w, hipStream_t st)
{
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idx, nullptr, w.seg, st);
    if (rc != DSV_OK) return rc;
    rc = launch_row_order(p, pl, w.seg, w.hist, w.order, st);
    if (rc != DSV_OK) return rc;
    {
        KernelSpan span(DSV_KERNEL_FWD_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            SplitPlan lp = pl;
            lp.nqb = (p.L + 256 / SweepLanes<T, D>::fwd - 1) / (256 / SweepLanes<T, D>::fwd);  // row blocks of this kernel's layout
            const int64_t blocks = (int64_t)tabs[t].n * lp.S_pad * lp.nqb;
            if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
            hipLaunchKernelGGL((sparse_fwd_split_kernel<T, D, SweepLanes<T, D>::fwd>), dim3((unsigned)blocks), dim3(256), 0, st, (const T *)Q,
                               (const T *)K, (const T *)V, idx, w.seg, w.order, w.pm, w.pl, w.pacc, p.L, p.scale, tabs[t], lp);
            DSV_LAUNCH_CHECK();
        }
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_fwd_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, w.pm,
                       w.pl, w.pacc, (T *)O, lse, n_rows, pl.S);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dq_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                 const void *K, const void *V, const int32_t *idx, const void *O, const float *lse,
                                 const void *dO, void *dQ, float *delta, const SplitPlan &pl,
                                 const BwdSplitWorkspace &w, hipStream_t st)
{
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idx, nullptr, w.seg, st);
    if (rc != DSV_OK) return rc;
    rc = launch_row_order(p, pl, w.seg, w.hist, w.order, st);
    if (rc != DSV_OK) return rc;
    {
        KernelSpan span(DSV_KERNEL_DQ_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            SplitPlan lp = pl;
            lp.nqb = (p.L + 256 / SweepLanes<T, D>::dq - 1) / (256 / SweepLanes<T, D>::dq);  // row blocks of this kernel's layout
            const int64_t blocks = (int64_t)tabs[t].n * lp.S_pad * lp.nqb;
            if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
            hipLaunchKernelGGL((sparse_bwd_dq_split_kernel<T, D, SweepLanes<T, D>::dq>), dim3((unsigned)blocks), dim3(256), 0, st, (const T *)Q,
                               (const T *)K, (const T *)V, idx, w.seg, w.order, (const T *)O, lse, (const T *)dO, w.pa, w.pb,
                               w.pdelta, p.L, p.scale, tabs[t], lp);
            DSV_LAUNCH_CHECK();
        }
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_bwd_dq_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, w.pa,
                       w.pb, w.pdelta, (const T *)O, (const T *)dO, (T *)dQ, delta, n_rows, pl.S, p.scale);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dkdv_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                   const void *K, const void *V, const int32_t *idxT, const int64_t *col,
                                   const float *lse, const float *delta, const void *dO, void *dK, void *dV,
                                   const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st, int expand_G)
{
    const int nbh = p.B * p.H;
    if (expand_G < 1 || (uint64_t)p.L * (uint64_t)expand_G >= (1ull << 32)) return DSV_EUNSUPPORTED;
    const GroupExpand ge = expand_G > 1 ? make_expand(expand_G) : no_expand();
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idxT, col, w.seg, st, ge);
    if (rc != DSV_OK) return rc;
    const int64_t nrows = (int64_t)nbh * p.L;
    hipLaunchKernelGGL(pack_rowstat_kernel, dim3((unsigned)((nrows + 255) / 256)), dim3(256), 0, st, lse, delta,
                       w.rowstat, nrows);
    DSV_LAUNCH_CHECK();
    rc = launch_row_order(p, pl, w.seg, w.hist, w.order, st);
    if (rc != DSV_OK) return rc;
    {
        KernelSpan span(DSV_KERNEL_DKDV_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            SplitPlan lp = pl;
            lp.nqb = (p.L + 256 / SweepLanes<T, D>::dkdv - 1) / (256 / SweepLanes<T, D>::dkdv);  // row blocks of this kernel's layout
            const int64_t blocks = (int64_t)tabs[t].n * lp.S_pad * lp.nqb;
            if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
            const size_t stat_bytes = (size_t)lp.range_len * sizeof(float2);  // <= kMaxRangeRows * 8
            auto kern = &sparse_bwd_dkdv_split_kernel<T, D, SweepLanes<T, D>::dkdv>;
            DSV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                              (int)(kMaxRangeRows * sizeof(float2))));
            hipLaunchKernelGGL(kern, dim3((unsigned)blocks), dim3(256), stat_bytes, st, (const T *)Q, (const T *)K,
                               (const T *)V, idxT, col, w.seg, w.order, (const float2 *)w.rowstat, (const T *)dO, w.pa, w.pb,
                               p.L, p.scale, tabs[t], lp, ge);
            DSV_LAUNCH_CHECK();
        }
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_bwd_dkdv_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st,
                       w.pa, w.pb, (T *)dK, (T *)dV, n_rows, pl.S, p.scale);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

// ---- pieces of the split plan used by the query-grouped kernels as well --------------------------------------
// Segment pointers of `rows` ascending index rows per head (tabs built for that many rows).
dsv_status launch_row_segments(const dsv_problem &p, int rows, const HeadTable *tabs, int n_tabs, const SplitPlan &pl,
                               const int32_t *index, int32_t *seg, hipStream_t st)
{
    const int64_t n = (int64_t)rows * (pl.S + 1);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((unsigned)((n + 255) / 256), tabs[t].n);
        hipLaunchKernelGGL(segment_ptr_kernel, grid, dim3(256), 0, st, index, (const int64_t *)nullptr, rows, tabs[t], pl, seg, no_expand());
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

// Merges of per-(token row, range) partials, bf16 d = 128 (the grouped kernels' case).
dsv_status launch_fwd_merge_bf16_128(const dsv_problem &p, const float *pm, const float *pl_, const float *pacc, void *O,
                                     float *lse, int S, hipStream_t st)
{
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_fwd_merge_kernel<bf16_t, 128>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, pm, pl_,
                       pacc, (bf16_t *)O, lse, n_rows, S);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_dq_merge_bf16_128(const dsv_problem &p, const float *pa, const float *pb, const float *pdelta,
                                    const void *O, const void *dO, void *dQ, float *delta, int S, hipStream_t st)
{
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_bwd_dq_merge_kernel<bf16_t, 128>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, pa, pb,
                       pdelta, (const bf16_t *)O, (const bf16_t *)dO, (bf16_t *)dQ, delta, n_rows, S, p.scale);
    DSV_LAUNCH_CHECK();
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

dsv_status launch_sparse_fwd_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                   const void *K, const void *V, const int32_t *idx, void *O, float *lse,
                                   const SplitPlan &pl, const FwdSplitWorkspace &w, hipStream_t st)
{
    DSV_DISPATCH_TD(fwd_split_t, p, tabs, n_tabs, Q, K, V, idx, O, lse, pl, w, st);
}

dsv_status launch_bwd_dq_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                               const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO,
                               void *dQ, float *delta, const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dq_split_t, p, tabs, n_tabs, Q, K, V, idx, O, lse, dO, dQ, delta, pl, w, st);
}

dsv_status launch_bwd_dkdv_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                 const void *K, const void *V, const int32_t *idxT, const int64_t *col,
                                 const float *lse, const float *delta, const void *dO, void *dK, void *dV,
                                 const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st, int expand_G)
{
    DSV_DISPATCH_TD(bwd_dkdv_split_t, p, tabs, n_tabs, Q, K, V, idxT, col, lse, delta, dO, dK, dV, pl, w, st, expand_G);
}

}  // namespace dsv
