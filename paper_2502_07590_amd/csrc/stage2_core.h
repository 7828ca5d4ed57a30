// Inner loops of stage 2, shared by the plain gather kernels (stage2.hip) and the L2-blocked
// kernels (stage2_split.hip).
//
// Lane layout: a group of LPR consecutive lanes (4, 8 or 16) owns one output row; lane s of the group
// holds CH = d/LPR channels of every [d]-vector, as 16-byte pieces taken from the s-th slot of every
// LPR*16-byte strip of the row (LaneLayout in common.h), so each load instruction of the group covers
// whole strips.  Fewer lanes per row mean more channels per lane: the per-pair bookkeeping (reductions,
// exponentials, weights, addresses) is shared by more arithmetic, at the price of more registers.
//
// Each sweep walks positions [tb, te) of one index row (or key-major list):
//   fwd_sweep   online softmax over the segment: running max m (log2 domain), l, acc = sum p v
//   dq_sweep    C = sum p (dP - D0) k,  B = sum p k,  Delta = sum p dP   (dP = dO . v; D0 = dO . O from
//               the stored O: a centring value within rounding of Delta, so that the weights of C are
//               the small, centred dS and survive bf16 rounding; dQ = scale (C - (Delta - D0) B))
//   dkdv_sweep  dK = sum dS q,   dV = sum p dO                            (dS = p (dP - Delta_i))
//
// bf16 rows: dots use v_dot2_f32_bf16 on the packed words; the accumulations "acc += w * row"
// take two gathered rows at a time, interleave their words with v_perm so that one packed word
// holds the same channel of both rows, and issue one v_dot2_f32_bf16 per channel with the two
// weights packed as bf16 -- half the VALU work of unpack + FMA.  The probabilities p are thereby
// rounded to bf16 (relative 2^-9, as any bf16 flash-attention kernel rounds P before its second
// GEMM); the signed, possibly large dS weights go in as two bf16 words (head + tail, 16
// significant bits, two dot2 per channel).  Accumulators stay fp32.  fp32 rows use plain FMAs.
#pragma once

#include "common.h"

namespace dsv {

// Lanes per row of each sweep (rows per 256-thread block = 256 / lanes), chosen through the bytes of a
// row each lane holds: 64 for the forward and the dkdv sweep, 32 for the dq sweep (it keeps three row
// chunks and two accumulators in registers).  Measured on MI355X at L = 128k, bf16, d = 128, k = 8192
// (ms per sweep): forward 16 lanes: 131, 8: 112, 4: 110; dq 16: 145, 8: 123, 4: 202 (registers);
// dkdv 16: 190, 8: 148, 4: 140.  Two steps per loop trip or 8 keys per forward step change nothing or
// cost a little (the gathers already fill the memory path).
#ifndef DSV_DQ_REP
#define DSV_DQ_REP 1
#endif
#ifndef DSV_DKDV_REP
#define DSV_DKDV_REP 1
#endif
#ifndef DSV_FWD_U
#define DSV_FWD_U 4   // keys per forward step (4 or 8)
#endif
#ifndef DSV_CHUNK_FWD
#define DSV_CHUNK_FWD 64
#endif
#ifndef DSV_CHUNK_DQ
#define DSV_CHUNK_DQ 32
#endif
#ifndef DSV_CHUNK_DKDV
#define DSV_CHUNK_DKDV 64
#endif
constexpr int lanes_for(int row_bytes, int chunk_bytes)
{
    const int l = row_bytes / chunk_bytes;
    return l < 4 ? 4 : (l > 16 ? 16 : l);
}
template <typename T, int D> struct SweepLanes {
    static constexpr int fwd = lanes_for(D * (int)sizeof(T), DSV_CHUNK_FWD);
    static constexpr int dq = lanes_for(D * (int)sizeof(T), DSV_CHUNK_DQ);
    static constexpr int dkdv = lanes_for(D * (int)sizeof(T), DSV_CHUNK_DKDV);
};

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

typedef __attribute__((__vector_size__(2 * sizeof(float)))) float floatx2_t;

// 2^x by the bare hardware instruction (denormal results flush to zero; arguments here are <= 0
// up to rounding, results are weights in [0, 1]).
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    floatx2_t f = {lo, hi};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, h);
}

// acc[c] += w_a * a[c] + w_b * b[c] for this lane's CH channels; wab = (bf16 w_a, bf16 w_b) packed
// (bf16 rows), or fa / fb the fp32 weights (fp32 rows).
template <typename T, int CH>
__device__ __forceinline__ void axpy_pair(float (&acc)[CH], const RowChunk<T, CH> &a, const RowChunk<T, CH> &b,
                                          float fa, float fb, uint32_t wab)
{
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            acc[c] = fmaf(fa, __uint_as_float(a.w[c]), acc[c]);
            acc[c] = fmaf(fb, __uint_as_float(b.w[c]), acc[c]);
        }
    } else {
        const bf16x2_t w = __builtin_bit_cast(bf16x2_t, wab);
#pragma unroll
        for (int i = 0; i < CH / 2; ++i) {
            const uint32_t lo = __builtin_amdgcn_perm(b.w[i], a.w[i], 0x05040100u);  // (a.ch[2i],   b.ch[2i])
            const uint32_t hi = __builtin_amdgcn_perm(b.w[i], a.w[i], 0x07060302u);  // (a.ch[2i+1], b.ch[2i+1])
            acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, lo), w, acc[2 * i], false);
            acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, hi), w, acc[2 * i + 1], false);
        }
    }
}

// A weight pair as two packed bf16 words whose sum carries 16 significant bits: w = head + tail.
// Used where the weights are signed and large (the centred dS terms): a single bf16 rounding of a
// weight of magnitude ~10 is an absolute error of ~0.02 in the accumulated gradient.
struct SplitWeights {
    uint32_t head, tail;
};
__device__ __forceinline__ SplitWeights split_weights(float wa, float wb)
{
    SplitWeights s;
    s.head = pack_bf16x2(wa, wb);
    s.tail = pack_bf16x2(wa - __uint_as_float(s.head << 16), wb - __uint_as_float(s.head & 0xFFFF0000u));
    return s;
}

// acc[c] += w_a * a[c] + w_b * b[c] with 16-bit weights (bf16 rows) or fp32 weights (fp32 rows).
template <typename T, int CH>
__device__ __forceinline__ void axpy_pair_precise(float (&acc)[CH], const RowChunk<T, CH> &a,
                                                  const RowChunk<T, CH> &b, float fa, float fb)
{
    if constexpr (sizeof(T) == 4) {
        axpy_pair<T, CH>(acc, a, b, fa, fb, 0u);
    } else {
        const SplitWeights w = split_weights(fa, fb);
        const bf16x2_t wh = __builtin_bit_cast(bf16x2_t, w.head), wt = __builtin_bit_cast(bf16x2_t, w.tail);
#pragma unroll
        for (int i = 0; i < CH / 2; ++i) {
            const bf16x2_t lo = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(b.w[i], a.w[i], 0x05040100u));
            const bf16x2_t hi = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(b.w[i], a.w[i], 0x07060302u));
            acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(lo, wt, acc[2 * i], false);
            acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(lo, wh, acc[2 * i], false);
            acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, wt, acc[2 * i + 1], false);
            acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, wh, acc[2 * i + 1], false);
        }
    }
}

// Two accumulators fed by the same pair of rows with different weights (dq sweep: C and B); the
// first weight pair (signed, centred dS terms) is applied with 16-bit weights, the second (the
// probabilities) with bf16 weights.
template <typename T, int CH>
__device__ __forceinline__ void axpy_pair2(float (&acc1)[CH], float (&acc2)[CH], const RowChunk<T, CH> &a,
                                           const RowChunk<T, CH> &b, float f1a, float f1b, float f2a, float f2b)
{
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const float av = __uint_as_float(a.w[c]), bv = __uint_as_float(b.w[c]);
            acc1[c] = fmaf(f1a, av, acc1[c]);
            acc1[c] = fmaf(f1b, bv, acc1[c]);
            acc2[c] = fmaf(f2a, av, acc2[c]);
            acc2[c] = fmaf(f2b, bv, acc2[c]);
        }
    } else {
        const SplitWeights w1s = split_weights(f1a, f1b);
        const bf16x2_t w1 = __builtin_bit_cast(bf16x2_t, w1s.head), w1t = __builtin_bit_cast(bf16x2_t, w1s.tail);
        const bf16x2_t w2 = __builtin_bit_cast(bf16x2_t, pack_bf16x2(f2a, f2b));
#pragma unroll
        for (int i = 0; i < CH / 2; ++i) {
            const bf16x2_t lo = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(b.w[i], a.w[i], 0x05040100u));
            const bf16x2_t hi = __builtin_bit_cast(bf16x2_t, __builtin_amdgcn_perm(b.w[i], a.w[i], 0x07060302u));
            acc1[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(lo, w1t, acc1[2 * i], false);
            acc1[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(lo, w1, acc1[2 * i], false);
            acc1[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, w1t, acc1[2 * i + 1], false);
            acc1[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, w1, acc1[2 * i + 1], false);
            acc2[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(lo, w2, acc2[2 * i], false);
            acc2[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(hi, w2, acc2[2 * i + 1], false);
        }
    }
}

// Row chunk of a gathered row: base is the head's [L, d] matrix (uniform across the wave), the
// per-lane part is a 32-bit element offset (row * D + the lane's LaneLayout offset), so the load can use a
// scalar base with a 32-bit vector offset.
template <typename T, int D, int LPR>
__device__ __forceinline__ RowChunk<T, D / LPR> gather_chunk(const T *__restrict__ head, uint32_t row, uint32_t lane_off)
{
    typedef LaneLayout<T, D, LPR> LL;
    const uint32_t byte_off = (row * (uint32_t)D + lane_off) * (uint32_t)sizeof(T);  // < 2^32: a head's matrix is < 4 GB
    return load_chunk<T, LL::CH, LL::PSB>(reinterpret_cast<const T *>(reinterpret_cast<const char *>(head) + byte_off));
}

// ------------------------------------------------------------------------------------ forward sweep
template <int CH> struct FwdState {
    float m, l;
    float acc[CH];
};

// jsrc: U staged index entries (LDS); TAIL: only the first nvalid of them count (the rest are valid
// row numbers too -- duplicates of the segment's last entry -- and get weight zero).
template <typename T, int D, int LPR, bool TAIL>
__device__ __forceinline__ void fwd_step(FwdState<D / LPR> &st, const RowChunk<T, D / LPR> &q, const T *__restrict__ Kh,
                                         const T *__restrict__ Vh, uint32_t lane_off, const int32_t *jsrc, int nvalid,
                                         float c2)
{
    constexpr int CH = D / LPR;
    constexpr int U = DSV_FWD_U;
    typedef RowChunk<T, CH> Chunk;
    int j[U];
    Chunk kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) j[u] = jsrc[u];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        kc[u] = gather_chunk<T, D, LPR>(Kh, (uint32_t)j[u], lane_off);
        vc[u] = gather_chunk<T, D, LPR>(Vh, (uint32_t)j[u], lane_off);
    }
    float sc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) sc[u] = dot_chunk<T, CH>(q, kc[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) sc[u] = row_sum<LPR>(sc[u]) * c2;
    if (TAIL) {
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (u >= nvalid) sc[u] = -INFINITY;
    }
    float mblk = fmaxf(fmaxf(sc[0], sc[1]), fmaxf(sc[2], sc[3]));
    if constexpr (U == 8) mblk = fmaxf(mblk, fmaxf(fmaxf(sc[4], sc[5]), fmaxf(sc[6], sc[7])));
    if (mblk > st.m) {  // rescale only when the running max moves (rare after the first blocks)
        const float corr = fast_exp2(st.m - mblk);
        st.m = mblk;
        st.l *= corr;
#pragma unroll
        for (int c = 0; c < CH; ++c) st.acc[c] *= corr;
    }
    float p[U];
#pragma unroll
    for (int u = 0; u < U; ++u) p[u] = fast_exp2(sc[u] - st.m);
#pragma unroll
    for (int u = 0; u < U; u += 4) st.l += (p[u] + p[u + 1]) + (p[u + 2] + p[u + 3]);
#pragma unroll
    for (int u = 0; u < U; u += 2)
        axpy_pair<T, CH>(st.acc, vc[u], vc[u + 1], p[u], p[u + 1], sizeof(T) == 2 ? pack_bf16x2(p[u], p[u + 1]) : 0u);
}

// ---- index staging ------------------------------------------------------------------------------
// The lanes of a group all need the same index entries.  Reading them straight from memory costs one
// full-width vector-memory instruction per step (as much address-path time as a whole gathered row)
// and re-fetches each 128-byte line of the row eight times through a cache that the gathers keep
// flushing.  Instead the group reads kStage entries at a time, each lane a different one (one
// coalesced request), parks them in its own slot of LDS, and the steps fetch them from there with
// 16-byte broadcast reads.  The next chunk is requested before the current one is consumed.
constexpr int kStage = 32;

template <int LPR> struct StagedIndex {
    static constexpr int EPL = kStage / LPR;  // entries each lane fetches per chunk
    int a[EPL];
    // request entries [c0, c0 + kStage) of `row`, clamped to the segment's last entry te - 1
    __device__ __forceinline__ void request(const int32_t *__restrict__ row, int c0, int te, int s)
    {
#pragma unroll
        for (int e = 0; e < EPL; ++e) a[e] = row[min(c0 + e * LPR + s, te - 1)];
    }
    // the same on the per-query list that a list of groups stands for
    __device__ __forceinline__ void request(const int32_t *__restrict__ row, int c0, int te, int s, const GroupExpand &ge)
    {
#pragma unroll
        for (int e = 0; e < EPL; ++e) a[e] = expanded_entry(row, min(c0 + e * LPR + s, te - 1), ge);
    }
    __device__ __forceinline__ void park(int32_t *stage, int s) const
    {
#pragma unroll
        for (int e = 0; e < EPL; ++e) stage[e * LPR + s] = a[e];
    }
};

// positions [tb, te) of `row`; all lanes of the group call with the same arguments.  stage: the
// group's kStage-entry LDS slot (16-byte aligned); s: this lane's number inside the group.
template <typename T, int D, int LPR>
__device__ __forceinline__ void fwd_sweep(FwdState<D / LPR> &st, const RowChunk<T, D / LPR> &q, const T *__restrict__ Kh,
                                          const T *__restrict__ Vh, uint32_t lane_off, const int32_t *__restrict__ row,
                                          int tb, int te, float c2, int32_t *stage, int s)
{
    if (tb >= te) return;
    StagedIndex<LPR> si;
    si.request(row, tb, te, s);
    for (int c0 = tb; c0 < te; c0 += kStage) {
        si.park(stage, s);
        if (c0 + kStage < te) si.request(row, c0 + kStage, te, s);
        const int n = min(kStage, te - c0);
        int it = 0;
        for (; it + DSV_FWD_U <= n; it += DSV_FWD_U) fwd_step<T, D, LPR, false>(st, q, Kh, Vh, lane_off, stage + it, DSV_FWD_U, c2);
        if (it < n) fwd_step<T, D, LPR, true>(st, q, Kh, Vh, lane_off, stage + it, n - it, c2);
    }
}

// ------------------------------------------------------------------------------------ dq sweep
template <int CH> struct DqState {
    float delta;
    float a[CH], b[CH];  // a: the centred sum C
};

template <typename T, int D, int LPR, bool TAIL>
__device__ __forceinline__ void dq_step(DqState<D / LPR> &st, const RowChunk<T, D / LPR> &q,
                                        const RowChunk<T, D / LPR> &go, const T *__restrict__ Kh,
                                        const T *__restrict__ Vh, uint32_t lane_off, const int32_t *jsrc, int nvalid,
                                        float c2, float lse2, float delta0)
{
    constexpr int CH = D / LPR;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    int j[U];
    Chunk kc[U], vc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) j[u] = jsrc[u];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        kc[u] = gather_chunk<T, D, LPR>(Kh, (uint32_t)j[u], lane_off);
        vc[u] = gather_chunk<T, D, LPR>(Vh, (uint32_t)j[u], lane_off);
    }
    float p[U], wc[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float sc = row_sum<LPR>(dot_chunk<T, CH>(q, kc[u]));
        const float dp = row_sum<LPR>(dot_chunk<T, CH>(go, vc[u]));
        p[u] = fast_exp2(sc * c2 - lse2);
        if (TAIL && u >= nvalid) p[u] = 0.f;
        st.delta = fmaf(p[u], dp, st.delta);
        wc[u] = p[u] * (dp - delta0);
    }
    axpy_pair2<T, CH>(st.a, st.b, kc[0], kc[1], wc[0], wc[1], p[0], p[1]);
}

template <typename T, int D, int LPR>
__device__ __forceinline__ void dq_sweep(DqState<D / LPR> &st, const RowChunk<T, D / LPR> &q,
                                         const RowChunk<T, D / LPR> &go, const T *__restrict__ Kh,
                                         const T *__restrict__ Vh, uint32_t lane_off, const int32_t *__restrict__ row,
                                         int tb, int te, float c2, float lse2, float delta0, int32_t *stage, int s)
{
    if (tb >= te) return;
    StagedIndex<LPR> si;
    si.request(row, tb, te, s);
    for (int c0 = tb; c0 < te; c0 += kStage) {
        si.park(stage, s);
        if (c0 + kStage < te) si.request(row, c0 + kStage, te, s);
        const int n = min(kStage, te - c0);
        int it = 0;
#if DSV_DQ_REP == 2
        for (; it + 4 <= n; it += 4) {
            dq_step<T, D, LPR, false>(st, q, go, Kh, Vh, lane_off, stage + it, 2, c2, lse2, delta0);
            dq_step<T, D, LPR, false>(st, q, go, Kh, Vh, lane_off, stage + it + 2, 2, c2, lse2, delta0);
        }
#endif
        for (; it + 2 <= n; it += 2) dq_step<T, D, LPR, false>(st, q, go, Kh, Vh, lane_off, stage + it, 2, c2, lse2, delta0);
        if (it < n) dq_step<T, D, LPR, true>(st, q, go, Kh, Vh, lane_off, stage + it, n - it, c2, lse2, delta0);
    }
}

// ------------------------------------------------------------------------------------ dkdv sweep
template <int CH> struct DkdvState {
    float dk[CH], dv[CH];
};

// stat_s (optional): the packed {lse * log2(e), Delta} entries of the queries from stat_base on, parked in
// LDS by the caller (every query of the list segment lies in that stretch); then lse_h / delta_h are unused.
template <typename T, int D, int LPR, bool TAIL, bool LDS_STAT>
__device__ __forceinline__ void dkdv_step(DkdvState<D / LPR> &st, const RowChunk<T, D / LPR> &kc,
                                          const RowChunk<T, D / LPR> &vc, const T *__restrict__ Qh,
                                          const T *__restrict__ Gh, const float *__restrict__ lse_h,
                                          const float *__restrict__ delta_h, const float2 *stat_s, int stat_base,
                                          uint32_t lane_off, const int32_t *jsrc, int nvalid, float c2)
{
    constexpr int CH = D / LPR;
    constexpr int U = 2;
    typedef RowChunk<T, CH> Chunk;
    int iq[U];
    Chunk qc[U], gc[U];
    float l2[U], dl[U];
#pragma unroll
    for (int u = 0; u < U; ++u) iq[u] = jsrc[u];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        qc[u] = gather_chunk<T, D, LPR>(Qh, (uint32_t)iq[u], lane_off);
        gc[u] = gather_chunk<T, D, LPR>(Gh, (uint32_t)iq[u], lane_off);
        if constexpr (LDS_STAT) {
            const float2 rs = stat_s[iq[u] - stat_base];
            l2[u] = rs.x;
            dl[u] = rs.y;
        } else if (delta_h) {
            l2[u] = lse_h[iq[u]] * kLog2e;
            dl[u] = delta_h[iq[u]];
        } else {  // lse_h is a packed array {lse * log2(e), Delta} per query: one 8-byte load
            const float2 rs = reinterpret_cast<const float2 *>(lse_h)[iq[u]];
            l2[u] = rs.x;
            dl[u] = rs.y;
        }
    }
    float p[U], ds[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float sc = row_sum<LPR>(dot_chunk<T, CH>(qc[u], kc));
        const float dp = row_sum<LPR>(dot_chunk<T, CH>(gc[u], vc));
        p[u] = fast_exp2(sc * c2 - l2[u]);
        if (TAIL && u >= nvalid) p[u] = 0.f;
        ds[u] = p[u] * (dp - dl[u]);
    }
    axpy_pair_precise<T, CH>(st.dk, qc[0], qc[1], ds[0], ds[1]);
    // dV of a popular key sums thousands of terms: bf16 weights alone would leave ~1e-2 of noise
    axpy_pair_precise<T, CH>(st.dv, gc[0], gc[1], p[0], p[1]);
}

template <typename T, int D, int LPR, bool LDS_STAT = false>
__device__ __forceinline__ void dkdv_sweep(DkdvState<D / LPR> &st, const RowChunk<T, D / LPR> &kc,
                                           const RowChunk<T, D / LPR> &vc, const T *__restrict__ Qh,
                                           const T *__restrict__ Gh, const float *__restrict__ lse_h,
                                           const float *__restrict__ delta_h, uint32_t lane_off,
                                           const int32_t *__restrict__ list, int tb, int te, float c2, int32_t *stage,
                                           int s, const float2 *stat_s = nullptr, int stat_base = 0,
                                           GroupExpand ge = no_expand())
{
    if (tb >= te) return;
    StagedIndex<LPR> si;
    si.request(list, tb, te, s, ge);
    for (int c0 = tb; c0 < te; c0 += kStage) {
        si.park(stage, s);
        if (c0 + kStage < te) si.request(list, c0 + kStage, te, s, ge);
        const int n = min(kStage, te - c0);
        int it = 0;
#if DSV_DKDV_REP == 2
        for (; it + 4 <= n; it += 4) {
            dkdv_step<T, D, LPR, false, LDS_STAT>(st, kc, vc, Qh, Gh, lse_h, delta_h, stat_s, stat_base, lane_off, stage + it, 2, c2);
            dkdv_step<T, D, LPR, false, LDS_STAT>(st, kc, vc, Qh, Gh, lse_h, delta_h, stat_s, stat_base, lane_off, stage + it + 2, 2, c2);
        }
#endif
        for (; it + 2 <= n; it += 2) dkdv_step<T, D, LPR, false, LDS_STAT>(st, kc, vc, Qh, Gh, lse_h, delta_h, stat_s, stat_base, lane_off, stage + it, 2, c2);
        if (it < n) dkdv_step<T, D, LPR, true, LDS_STAT>(st, kc, vc, Qh, Gh, lse_h, delta_h, stat_s, stat_base, lane_off, stage + it, n - it, c2);
    }
}

}  // namespace dsv
