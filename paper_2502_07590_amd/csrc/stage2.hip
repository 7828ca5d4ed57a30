// Stage 2: exact softmax attention over the selected KV only, forward and backward
// (paper Sec. "Sparse Attention with Query Grouping", per-query form; attention formula of
// Sec. "Various Self-Attention Paradigms").
//
// Work layout shared by the kernels here: a group of 16 lanes (one DPP row) owns one query row;
// lane s of the group holds channels [s*CH, (s+1)*CH) of every [d]-vector, CH = d/16, so one
// wave-wide load instruction fetches four whole K (or V) rows as four contiguous segments.
// Dot products are reduced inside the row with DPP rotations.  A wave handles 4 queries, a block
// 16 consecutive queries of one head.
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
// Query-major pass: recomputes p and dS per selected pair, accumulates dQ in registers and adds
// the pair's contributions to fp32 dK / dV accumulators with hardware float atomics.
template <typename T, int D>
__global__ __launch_bounds__(256) void sparse_bwd_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                         const T *__restrict__ V, const int32_t *__restrict__ idx,
                                                         const T *__restrict__ O, const float *__restrict__ lse,
                                                         const T *__restrict__ dO, T *__restrict__ dQ,
                                                         float *__restrict__ dKacc, float *__restrict__ dVacc, int L,
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
    float *dKb = dKacc + head_base + s * CH;
    float *dVb = dVacc + head_base + s * CH;
    const int32_t *row = idx + tab.off[slot] + i * k;

    const Chunk q = load_chunk<T, CH>(Q + head_base + i * D + s * CH);
    const Chunk go = load_chunk<T, CH>(dO + head_base + i * D + s * CH);
    const Chunk o = load_chunk<T, CH>(O + head_base + i * D + s * CH);
    float qf[CH], gof[CH], of[CH];
    unpack_chunk<T, CH>(q, qf);
    unpack_chunk<T, CH>(go, gof);
    unpack_chunk<T, CH>(o, of);
    float delta = 0.f;
#pragma unroll
    for (int c = 0; c < CH; ++c) delta = fmaf(gof[c], of[c], delta);
    delta = row16_sum(delta);
    const float c2 = scale * kLog2e;
    const float lse2 = lse[(int64_t)bh * L + i] * kLog2e;

    float dq[CH];
#pragma unroll
    for (int c = 0; c < CH; ++c) dq[c] = 0.f;

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
            const bool on = live && (t0 + u < k);
            const float p = on ? exp2f(sc * c2 - lse2) : 0.f;
            const float ds = p * (dp - delta);
            float kf[CH];
            unpack_chunk<T, CH>(kc[u], kf);
#pragma unroll
            for (int c = 0; c < CH; ++c) dq[c] = fmaf(ds, kf[c], dq[c]);
            if (on) {
                const float dss = ds * scale;
                float *dkp = dKb + (int64_t)j[u] * D;
                float *dvp = dVb + (int64_t)j[u] * D;
#pragma unroll
                for (int c = 0; c < CH; ++c) {
                    unsafeAtomicAdd(dkp + c, dss * qf[c]);
                    unsafeAtomicAdd(dvp + c, p * gof[c]);
                }
            }
        }
    }
    if (live) {
#pragma unroll
        for (int c = 0; c < CH; ++c) dq[c] *= scale;
        store_chunk<T, CH>(dQ + head_base + i * D + s * CH, dq);
    }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(float4 *__restrict__ p, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n4; e += stride)
        p[e] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// fp32 accumulators -> output type, 4 elements per thread.
template <typename T>
__global__ __launch_bounds__(256) void convert_out_kernel(const float4 *__restrict__ a, const float4 *__restrict__ b,
                                                          T *__restrict__ oa, T *__restrict__ ob, int64_t n4)
{
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < n4; e += stride) {
        const float4 x = a[e], y = b[e];
        const float xf[4] = {x.x, x.y, x.z, x.w}, yf[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            oa[4 * e + c] = from_f32<T>(xf[c]);
            ob[4 * e + c] = from_f32<T>(yf[c]);
        }
    }
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
static dsv_status bwd_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                        const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO, void *dQ,
                        void *dK, void *dV, float *dKacc, float *dVacc, hipStream_t st)
{
    const int64_t n = (int64_t)p.B * p.H * p.L * p.d;  // multiple of 64
    const int64_t n4 = n / 4;
    const int fill_blocks = (int)((n4 + 255) / 256 < 4096 ? (n4 + 255) / 256 : 4096);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(fill_blocks), dim3(256), 0, st, (float4 *)dKacc, n4);
    hipLaunchKernelGGL(fill_zero_kernel, dim3(fill_blocks), dim3(256), 0, st, (float4 *)dVacc, n4);
    DSV_LAUNCH_CHECK();
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid((p.L + 15) / 16, tabs[t].n);
        hipLaunchKernelGGL((sparse_bwd_kernel<T, D>), grid, dim3(256), 0, st, (const T *)Q, (const T *)K, (const T *)V,
                           idx, (const T *)O, lse, (const T *)dO, (T *)dQ, dKacc, dVacc, p.L, p.scale, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    hipLaunchKernelGGL((convert_out_kernel<T>), dim3(fill_blocks), dim3(256), 0, st, (const float4 *)dKacc,
                       (const float4 *)dVacc, (T *)dK, (T *)dV, n4);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_sparse_bwd(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO,
                             void *dQ, void *dK, void *dV, float *dKacc, float *dVacc, hipStream_t st)
{
#define DSV_CASE(TT, DD) \
    return bwd_t<TT, DD>(p, tabs, n_tabs, Q, K, V, idx, O, lse, dO, dQ, dK, dV, dKacc, dVacc, st)
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) DSV_CASE(bf16_t, 64);
        if (p.d == 128) DSV_CASE(bf16_t, 128);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) DSV_CASE(float, 64);
        if (p.d == 128) DSV_CASE(float, 128);
    }
#undef DSV_CASE
    return DSV_EUNSUPPORTED;
}

}  // namespace dsv
