// Stage 2, L2-blocked form, for index rows (and key-major lists) in ascending order.
//
// The plain gather kernels (stage2.hip) fetch every selected K/V row from wherever it lives; at
// L = 128k a head's K+V slab is 67 MB, far beyond the 4 MB L2 of an XCD, so the gathers are served
// by the memory-side cache at about its bandwidth.  Here the key axis is cut into ranges whose K+V
// rows fit one XCD's L2 with room to spare.  Because a row of idx is ascending, the keys a query
// selected inside one range are one contiguous segment of its row.  Work item = (head, range,
// block of 16 queries); the 1-D grid is laid out so that workgroup b runs on XCD b % 8 and every
// XCD walks "its" ranges one after the other with all of its CUs inside the same range, which
// keeps that range's rows resident in that XCD's L2.  Each item leaves a partial result per query
// (split-K); a small second kernel merges the partials.
//
// Same lane layout as stage2.hip: 16 lanes per query, lane s holds channels [s*CH, (s+1)*CH).
#include <algorithm>

#include "common.h"

namespace dsv {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Decode a linear block id into (head slot, range, query block).  Consecutive ids go to
// consecutive XCDs; ids b, b+8, b+16, ... (one XCD) walk the query blocks of one range, then the
// next range of that XCD.  Ranges are padded to a multiple of 8; padded ranges return false.
__device__ __forceinline__ bool decode_item(const SplitPlan &pl, int64_t b, int &slot, int &range, int &qb)
{
    const int64_t per_head = (int64_t)pl.S_pad * pl.nqb;
    slot = (int)(b / per_head);
    const int64_t rem = b - (int64_t)slot * per_head;
    const int xcd = (int)(rem & 7);
    const int64_t local = rem >> 3;
    const int t = (int)(local / pl.nqb);
    qb = (int)(local - (int64_t)t * pl.nqb);
    range = t * 8 + xcd;
    return range < pl.S;
}

// ---- segment pointers -----------------------------------------------------------------------
// seg[bh, row, s] = first position in the (ascending) row whose value is >= s * range_len, for
// s = 0 .. S.  Query-major: rows of idx (length k).  Key-major: lists of idx_t (start and length
// from col_ptr), cut by QUERY ranges.
__global__ __launch_bounds__(256) void segment_ptr_kernel(const int32_t *__restrict__ index, const int64_t *__restrict__ col,
                                                          int L, HeadTable tab, SplitPlan pl,
                                                          int32_t *__restrict__ seg)
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
        len = (int)(cp[row + 1] - cp[row]);
    } else {
        len = tab.k[slot];
        base = index + tab.off[slot] + (int64_t)row * len;
    }
    const int64_t target = (int64_t)s * pl.range_len;
    int lo = 0, hi = len;  // first position with value >= target
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if ((int64_t)base[mid] < target) lo = mid + 1; else hi = mid;
    }
    seg[((int64_t)bh * L + row) * np + s] = lo;
}

// ---- forward ----------------------------------------------------------------------------------
// Partial softmax state of one (query, range): running max m (log2 domain), l = sum 2^(s-m),
// acc = sum 2^(s-m) v.  Empty segments leave (m = -inf, l = 0, acc = 0).
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_fwd_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                               const T *__restrict__ V,
                                                               const int32_t *__restrict__ idx,
                                                               const int32_t *__restrict__ seg, float *__restrict__ pm,
                                                               float *__restrict__ pl_, float *__restrict__ pacc, int L,
                                                               float scale, HeadTable tab, SplitPlan pl)
{
    constexpr int CH = D / 16;
    constexpr int U = 4;
    typedef RowChunk<T, CH> Chunk;
    int slot, range, qb;
    if (!decode_item(pl, blockIdx.x, slot, range, qb)) return;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t iq = (int64_t)qb * 16 + wave * 4 + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Kb = K + head_base + s * CH;
    const T *Vb = V + head_base + s * CH;
    const int32_t *row = idx + tab.off[slot] + i * k;
    const int32_t *sp = seg + ((int64_t)bh * L + i) * (pl.S + 1) + range;
    const int tb = sp[0], te = sp[1];

    const Chunk q = load_chunk<T, CH>(Q + head_base + i * D + s * CH);
    const float c2 = scale * kLog2e;
    float m = -INFINITY, l = 0.f;
    float acc[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) acc[c] = 0.f;

    for (int t0 = tb; t0 < te; t0 += U) {
        int j[U];
        Chunk kc[U], vc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) j[u] = row[min(t0 + u, te - 1)];
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
            if (t0 + u >= te) sc[u] = -INFINITY;
        float mnew = m;
#pragma unroll
        for (int u = 0; u < U; ++u) mnew = fmaxf(mnew, sc[u]);
        const float corr = exp2f(m - mnew);
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
    if (live) {
        const int64_t slot_id = ((int64_t)bh * L + i) * pl.S + range;
        store_chunk<float, CH>(pacc + slot_id * D + s * CH, acc);
        if (s == 0) { pm[slot_id] = m; pl_[slot_id] = l; }
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
// Per (query, key range): A = sum p dP k, B = sum p k, Delta = sum p dP over the segment (all three
// are plain sums over the selected keys, so partials simply add).
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dq_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                  const T *__restrict__ V,
                                                                  const int32_t *__restrict__ idx,
                                                                  const int32_t *__restrict__ seg,
                                                                  const float *__restrict__ lse,
                                                                  const T *__restrict__ dO, float *__restrict__ pa,
                                                                  float *__restrict__ pb, float *__restrict__ pdelta,
                                                                  int L, float scale, HeadTable tab, SplitPlan pl)
{
    constexpr int CH = D / 16;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    int slot, range, qb;
    if (!decode_item(pl, blockIdx.x, slot, range, qb)) return;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t iq = (int64_t)qb * 16 + wave * 4 + grp;
    const bool live = iq < L;
    const int64_t i = live ? iq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Kb = K + head_base + s * CH;
    const T *Vb = V + head_base + s * CH;
    const int32_t *row = idx + tab.off[slot] + i * k;
    const int32_t *sp = seg + ((int64_t)bh * L + i) * (pl.S + 1) + range;
    const int tb = sp[0], te = sp[1];

    const Chunk q = load_chunk<T, CH>(Q + head_base + i * D + s * CH);
    const Chunk go = load_chunk<T, CH>(dO + head_base + i * D + s * CH);
    const float c2 = scale * kLog2e;
    const float lse2 = lse[(int64_t)bh * L + i] * kLog2e;

    float a[CH], bsum[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { a[c] = 0.f; bsum[c] = 0.f; }
    float delta = 0.f;

    for (int t0 = tb; t0 < te; t0 += U) {
        int j[U];
        Chunk kc[U], vc[U];
#pragma unroll
        for (int u = 0; u < U; ++u) j[u] = row[min(t0 + u, te - 1)];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            kc[u] = load_chunk<T, CH>(Kb + (int64_t)j[u] * D);
            vc[u] = load_chunk<T, CH>(Vb + (int64_t)j[u] * D);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float sc = row16_sum(dot_chunk<T, CH>(q, kc[u]));
            const float dp = row16_sum(dot_chunk<T, CH>(go, vc[u]));
            const float p = (t0 + u < te) ? exp2f(sc * c2 - lse2) : 0.f;
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
        const int64_t slot_id = ((int64_t)bh * L + i) * pl.S + range;
        store_chunk<float, CH>(pa + slot_id * D + s * CH, a);
        store_chunk<float, CH>(pb + slot_id * D + s * CH, bsum);
        if (s == 0) pdelta[slot_id] = delta;
    }
}

// dQ_i = scale * (sum_s A_s - Delta_i * sum_s B_s), Delta_i = sum_s Delta_s.
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dq_merge_kernel(const float *__restrict__ pa,
                                                                  const float *__restrict__ pb,
                                                                  const float *__restrict__ pdelta,
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
    float dq[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) dq[c] = scale * (a[c] - delta * b[c]);
    store_chunk<T, CH>(dQ + row * D + s * CH, dq);
    if (s == 0) delta_out[row] = delta;
}

// ---- backward, dkdv step -------------------------------------------------------------------------
// Key-major: work item = (head, QUERY range, block of 16 keys); a key's ascending query list has one
// contiguous segment per query range, whose Q / dO rows (and lse, Delta entries) stay in L2.
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_dkdv_split_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                    const T *__restrict__ V,
                                                                    const int32_t *__restrict__ idxT,
                                                                    const int64_t *__restrict__ col,
                                                                    const int32_t *__restrict__ seg,
                                                                    const float *__restrict__ lse,
                                                                    const float *__restrict__ delta,
                                                                    const T *__restrict__ dO, float *__restrict__ pdk,
                                                                    float *__restrict__ pdv, int L, float scale,
                                                                    HeadTable tab, SplitPlan pl)
{
    constexpr int CH = D / 16;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    int slot, range, kb;
    if (!decode_item(pl, blockIdx.x, slot, range, kb)) return;
    const int bh = tab.bh[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int grp = lane >> 4, s = lane & 15;
    const int64_t jq = (int64_t)kb * 16 + wave * 4 + grp;
    const bool live = jq < L;
    const int64_t j = live ? jq : L - 1;
    const int64_t head_base = (int64_t)bh * L * D;
    const T *Qb = Q + head_base + s * CH;
    const T *Gb = dO + head_base + s * CH;
    const float *lse_b = lse + (int64_t)bh * L;
    const float *delta_b = delta + (int64_t)bh * L;
    const int32_t *list = idxT + tab.off[slot] + col[(int64_t)bh * (L + 1) + j];
    const int32_t *sp = seg + ((int64_t)bh * L + j) * (pl.S + 1) + range;
    const int tb = sp[0], te = live ? sp[1] : sp[0];

    const Chunk kc = load_chunk<T, CH>(K + head_base + j * D + s * CH);
    const Chunk vc = load_chunk<T, CH>(V + head_base + j * D + s * CH);
    const float c2 = scale * kLog2e;
    float dk[CH], dv[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) { dk[c] = 0.f; dv[c] = 0.f; }

    for (int t0 = tb; t0 < te; t0 += U) {
        int iq[U];
        Chunk qc[U], gc[U];
        float l2[U], dl[U];
#pragma unroll
        for (int u = 0; u < U; ++u) iq[u] = list[min(t0 + u, te - 1)];
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
            const float p = (t0 + u < te) ? exp2f(sc * c2 - l2[u]) : 0.f;
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
        const int64_t slot_id = ((int64_t)bh * L + j) * pl.S + range;
        store_chunk<float, CH>(pdk + slot_id * D + s * CH, dk);
        store_chunk<float, CH>(pdv + slot_id * D + s * CH, dv);
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

// ------------------------------------------------------------------------------------ host
SplitPlan make_split_plan(const dsv_problem &p)
{
    const size_t esz = p.dtype == DSV_BF16 ? 2 : 4;
    const size_t row_pair_bytes = 2 * (size_t)p.d * esz;  // one K row + one V row (or Q + dO)
    SplitPlan pl;
    pl.range_len = (int)std::max<size_t>(256, kSplitRangeBytes / row_pair_bytes);
    pl.S = (p.L + pl.range_len - 1) / pl.range_len;
    pl.S_pad = (pl.S + 7) / 8 * 8;
    pl.nqb = (p.L + 15) / 16;
    return pl;
}

static dsv_status launch_segments(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const SplitPlan &pl,
                                  const int32_t *index, const int64_t *col, int32_t *seg, hipStream_t st)
{
    const int64_t n = (int64_t)p.L * (pl.S + 1);
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((unsigned)((n + 255) / 256), tabs[t].n);
        hipLaunchKernelGGL(segment_ptr_kernel, grid, dim3(256), 0, st, index, col, p.L, tabs[t], pl, seg);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

template <typename T, int D>
static dsv_status fwd_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                              const void *V, const int32_t *idx, void *O, float *lse, const SplitPlan &pl,
                              const FwdSplitWorkspace &w, hipStream_t st)
{
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idx, nullptr, w.seg, st);
    if (rc != DSV_OK) return rc;
    for (int t = 0; t < n_tabs; ++t) {
        const int64_t blocks = (int64_t)tabs[t].n * pl.S_pad * pl.nqb;
        if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
        hipLaunchKernelGGL((sparse_fwd_split_kernel<T, D>), dim3((unsigned)blocks), dim3(256), 0, st, (const T *)Q,
                           (const T *)K, (const T *)V, idx, w.seg, w.pm, w.pl, w.pacc, p.L, p.scale, tabs[t], pl);
        DSV_LAUNCH_CHECK();
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_fwd_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, w.pm,
                       w.pl, w.pacc, (T *)O, lse, n_rows, pl.S);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_sparse_fwd_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                   const void *K, const void *V, const int32_t *idx, void *O, float *lse,
                                   const SplitPlan &pl, const FwdSplitWorkspace &w, hipStream_t st)
{
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) return fwd_split_t<bf16_t, 64>(p, tabs, n_tabs, Q, K, V, idx, O, lse, pl, w, st);
        if (p.d == 128) return fwd_split_t<bf16_t, 128>(p, tabs, n_tabs, Q, K, V, idx, O, lse, pl, w, st);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) return fwd_split_t<float, 64>(p, tabs, n_tabs, Q, K, V, idx, O, lse, pl, w, st);
        if (p.d == 128) return fwd_split_t<float, 128>(p, tabs, n_tabs, Q, K, V, idx, O, lse, pl, w, st);
    }
    return DSV_EUNSUPPORTED;
}

template <typename T, int D>
static dsv_status bwd_dq_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                 const void *K, const void *V, const int32_t *idx, const float *lse, const void *dO,
                                 void *dQ, float *delta, const SplitPlan &pl, const BwdSplitWorkspace &w,
                                 hipStream_t st)
{
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idx, nullptr, w.seg, st);
    if (rc != DSV_OK) return rc;
    for (int t = 0; t < n_tabs; ++t) {
        const int64_t blocks = (int64_t)tabs[t].n * pl.S_pad * pl.nqb;
        if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
        hipLaunchKernelGGL((sparse_bwd_dq_split_kernel<T, D>), dim3((unsigned)blocks), dim3(256), 0, st, (const T *)Q,
                           (const T *)K, (const T *)V, idx, w.seg, lse, (const T *)dO, w.pa, w.pb, w.pdelta, p.L,
                           p.scale, tabs[t], pl);
        DSV_LAUNCH_CHECK();
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_bwd_dq_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st, w.pa,
                       w.pb, w.pdelta, (T *)dQ, delta, n_rows, pl.S, p.scale);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status bwd_dkdv_split_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                   const void *K, const void *V, const int32_t *idxT, const int64_t *col,
                                   const float *lse, const float *delta, const void *dO, void *dK, void *dV,
                                   const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st)
{
    dsv_status rc = launch_segments(p, tabs, n_tabs, pl, idxT, col, w.seg, st);
    if (rc != DSV_OK) return rc;
    for (int t = 0; t < n_tabs; ++t) {
        const int64_t blocks = (int64_t)tabs[t].n * pl.S_pad * pl.nqb;
        if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
        hipLaunchKernelGGL((sparse_bwd_dkdv_split_kernel<T, D>), dim3((unsigned)blocks), dim3(256), 0, st,
                           (const T *)Q, (const T *)K, (const T *)V, idxT, col, w.seg, lse, delta, (const T *)dO, w.pa,
                           w.pb, p.L, p.scale, tabs[t], pl);
        DSV_LAUNCH_CHECK();
    }
    const int64_t n_rows = (int64_t)p.B * p.H * p.L;
    hipLaunchKernelGGL((sparse_bwd_dkdv_merge_kernel<T, D>), dim3((unsigned)((n_rows + 15) / 16)), dim3(256), 0, st,
                       w.pa, w.pb, (T *)dK, (T *)dV, n_rows, pl.S, p.scale);
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

dsv_status launch_bwd_dq_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                               const void *V, const int32_t *idx, const float *lse, const void *dO, void *dQ,
                               float *delta, const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dq_split_t, p, tabs, n_tabs, Q, K, V, idx, lse, dO, dQ, delta, pl, w, st);
}

dsv_status launch_bwd_dkdv_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                 const void *K, const void *V, const int32_t *idxT, const int64_t *col,
                                 const float *lse, const float *delta, const void *dO, void *dK, void *dV,
                                 const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st)
{
    DSV_DISPATCH_TD(bwd_dkdv_split_t, p, tabs, n_tabs, Q, K, V, idxT, col, lse, delta, dO, dK, dV, pl, w, st);
}

}  // namespace dsv
