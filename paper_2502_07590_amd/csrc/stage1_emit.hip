// Stage 1, emission: once every query's threshold score tau and its tie budget are known
// (stage1.hip), write the selected keys of every query (idx, query-major) and, on request, the
// selecting queries of every key (idx_t, key-major).  Both are pure re-evaluations of
//   selected(i, j)  <=>  s_ij > tau_i  or  (s_ij == tau_i and j <= jcut_i)
// over recomputed score tiles; jcut_i is the index of the last threshold-equal key query i takes
// (lowest index first), or kAllTies when it takes all of them -- then "s_ij >= tau_i" decides, which
// is the case for every query unless scores tie exactly at the threshold.
//
// Layout of both kernels: one wave owns 32 "owners" (queries for idx, keys for idx_t) as the MFMA
// column operand and walks the other axis in tiles of 32, ascending.  Lanes l and l+32 hold the same
// owner; each has 16 predicate bits, which are merged into one 32-bit mask in ascending order of the
// other axis.  The masks are parked in LDS and expanded into index entries in batches (below), in tile
// order, so every row / list comes out ascending without any sorting.
#include "stage1_core.h"

namespace dsv {

// 16 predicate bits of a lane, bit tile_pos(v) <- pred(v); the caller shifts by 4*half and merges.
#define DSV_MASK16(m, pred_expr)                                   \
    do {                                                           \
        (m) = 0u;                                                  \
        _Pragma("unroll") for (int v = 0; v < 16; ++v)             \
            (m) |= (uint32_t)(pred_expr) << tile_pos(v);           \
    } while (0)

// Same, for predicates of the form "d(v) < 0" with d a float expression (NaN-free): the sign bits
// are shifted into a register with one v_alignbit each (no compare, no condition-code traffic),
// then put in tile order: bit-reverse, and spread the four nibbles to the low nibbles of four bytes.
#define DSV_SIGNMASK16(m, d_expr)                                                          \
    do {                                                                                   \
        uint32_t acc_ = 0u;                                                                \
        _Pragma("unroll") for (int v = 0; v < 16; ++v)                                     \
            acc_ = __builtin_amdgcn_alignbit(acc_, __float_as_uint(d_expr), 31);           \
        acc_ = __builtin_bitreverse32(acc_) >> 16; /* bit v = sign of d(v) */              \
        acc_ = (acc_ | (acc_ << 8)) & 0x00FF00FFu;                                         \
        (m) = (acc_ | (acc_ << 4)) & 0x0F0F0F0Fu;  /* bit tile_pos(v) */                   \
    } while (0)

__device__ __forceinline__ uint32_t merge_halves(uint32_t m, int half)
{
    m <<= 4 * half;
    return m | (uint32_t)__shfl_xor((int)m, 32);
}

// ---- output: masks parked per tile, expanded in batches -------------------------------------------
// A selected entry is 4 bytes and consecutive entries of one owner are produced ~16 tiles apart, so
// writing them as they appear makes every store a partial cache line (measured: 5x write
// amplification), and appending them one by one to a per-owner buffer costs a serial loop per tile
// that runs as long as the fullest of the 32 owners needs.  Instead the wave parks each tile's 32-bit
// mask per owner in LDS and, every kBatch tiles, expands owner by owner: the 32 lanes of a half-wave
// take the owner's 32 parked words (one tile each), a prefix sum of their popcounts gives every lane its
// place in the owner's row, and the lanes write their entries side by side -- one store instruction
// covers a contiguous stretch of the row.  Two owners are expanded at a time (one per half-wave).
constexpr int kBatch = 32;  // tiles between two expansions (= lanes of a half-wave)

struct OwnerOut {
    int64_t off;    // where the owner's row / list starts: element offset inside the index array (an offset, not
                    // a pointer: a pointer read back from LDS has lost its address space and would make every
                    // store a flat one)
    int32_t wpos;   // entries written so far
    int32_t limit;  // entries the row may hold (a correct threshold fills it exactly; the clamp keeps a
                    // wrong one from writing out of bounds)
};

struct EmitShared {
    uint32_t mask[kBatch][33];  // [tile in batch][owner], padded: conflict-free both ways
    OwnerOut out[32];
};

// inclusive prefix sum inside each half-wave (lanes 0..31 and lanes 32..63 separately)
__device__ __forceinline__ int half_scan(int x)
{
    int s = x;
    s += __builtin_amdgcn_update_dpp(0, s, 0x111, 0xF, 0xF, false);  // row_shr:1 (rows of 16 lanes, zero fill)
    s += __builtin_amdgcn_update_dpp(0, s, 0x112, 0xF, 0xF, false);  // row_shr:2
    s += __builtin_amdgcn_update_dpp(0, s, 0x114, 0xF, 0xF, false);  // row_shr:4
    s += __builtin_amdgcn_update_dpp(0, s, 0x118, 0xF, 0xF, false);  // row_shr:8
    s += __builtin_amdgcn_update_dpp(0, s, 0x142, 0xA, 0xF, false);  // row_bcast15 into rows 1 and 3
    return s;
}

// Expand the parked masks of tiles tile0 .. tile0 + nfilled - 1 for all 32 owners.
// (Compacting an owner's entries in LDS first and writing them out with consecutive lanes on consecutive
// entries was measured slower -- 24.2 against 21.2 ms for the query-major emission at L = 128k, k = 8192 --:
// the stores are not what bounds this loop.)
__device__ __forceinline__ void expand_batch(EmitShared &sh, int32_t *__restrict__ out, int tile0, int nfilled, int lane)
{
    const int t = lane & 31, half = lane >> 5;
    const int base_val = (tile0 + t) * 32;
    for (int o0 = 0; o0 < 32; o0 += 2) {
        const int o = o0 + half;
        uint32_t m = t < nfilled ? sh.mask[t][o] : 0u;
        const int c = __popc(m);
        const int incl = half_scan(c);
        const OwnerOut oo = sh.out[o];
        const int pos = oo.wpos + incl - c;
        if (pos + c > oo.limit) {  // entries past the row's capacity are dropped, highest first
            const int room = max(oo.limit - pos, 0);
            while (__popc(m) > room) m &= ~(0x80000000u >> __clz(m));
        }
        int32_t *dst = out + oo.off + pos;
        while (m) {  // each lane walks its own word; the wave leaves when the fullest word is done
            *dst++ = base_val + (__ffs(m) - 1);
            m &= m - 1;
        }
        if (t == 31) sh.out[o].wpos = min(oo.wpos + incl, oo.limit);
    }
}

// ------------------------------------------------------------------------------------ query-major
// prefix[query] holds the order-preserving key of tau on entry and the fp32 bits of tau on exit.
// krem[query] = +-(number of threshold-equal keys to take); negative: that is all of them.
// jcut (optional) and tile_flag (optional; 1 when all 32 queries of the tile take all their ties)
// are what the key-major emission needs.
template <typename T, int R>
__global__ __launch_bounds__(64) void emit_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq, int L,
                                                  HeadTable tab, uint32_t *__restrict__ prefix,
                                                  const int32_t *__restrict__ krem, int32_t *__restrict__ idx,
                                                  int32_t *__restrict__ jcut, int32_t *__restrict__ tile_flag)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * Lq * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x;
    const int n = lane & 31, half = lane >> 5;
    const bool live = q0 + n < Lq;
    const int qi = min(q0 + n, Lq - 1);
    const int64_t g = (int64_t)bh * padded_len(Lq) + qi;
    const float tau = key_score(prefix[g]);
    const int kr = krem[g];
    const int ties_wanted = kr < 0 ? -kr : kr;
    const bool all_simple = __all(kr < 0);
    const int64_t row_off = tab.off[slot] + (int64_t)qi * k;

    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, Lq, lane);
    __shared__ __align__(16) EmitShared sh;
    if (half == 0) sh.out[n] = OwnerOut{row_off, 0, live ? k : 0};
    int ties_taken = 0, last_tie = -1;
    const int ntiles = (L + 31) >> 5;
    Frag<T, R> kf_next = load_frag<T, R>(Kb, 0, L, lane);
    for (int tile = 0; tile < ntiles; ++tile) {
        const int j0 = tile * 32;
        // the next tile's fragment is requested before this tile is scored (rows past the end clamp)
        const Frag<T, R> kf = kf_next;
        kf_next = load_frag<T, R>(Kb, j0 + 32, L, lane);
        const floatx16_t acc = score_tile<T, R>(kf, qf);
        const uint32_t valid = (j0 + 32 <= L) ? 0xFFFFFFFFu : ((1u << (L - j0)) - 1u);
        uint32_t sel;
        if (all_simple) {
            uint32_t mlt;  // score < tau  <=>  (score - tau) is negative; equal scores give +0
            DSV_SIGNMASK16(mlt, acc[v] - tau);
            sel = ~merge_halves(mlt, half) & valid;
        } else {
            uint32_t mgt, meq;
            DSV_MASK16(mgt, acc[v] > tau);
            DSV_MASK16(meq, acc[v] == tau);
            mgt = merge_halves(mgt, half) & valid;
            meq = merge_halves(meq, half) & valid;
            if (meq) {
                const int room = ties_wanted - ties_taken;
                while (__popc(meq) > room) meq &= ~(0x80000000u >> __clz(meq));  // drop the highest index
                ties_taken += __popc(meq);
                if (meq) last_tie = j0 + 31 - __clz(meq);
            }
            sel = mgt | meq;
        }
        if (!live) sel = 0u;
        if (half == 0) sh.mask[tile % kBatch][n] = sel;
        if (tile % kBatch == kBatch - 1) expand_batch(sh, idx, tile - (kBatch - 1), kBatch, lane);
    }
    if (ntiles % kBatch) expand_batch(sh, idx, ntiles - ntiles % kBatch, ntiles % kBatch, lane);
    if (live && half == 0) {
        prefix[g] = __float_as_uint(tau);
        if (jcut) jcut[g] = kr < 0 ? kAllTies : last_tie;
    }
    if (tile_flag && lane == 0) tile_flag[(int64_t)bh * gridDim.x + blockIdx.x] = all_simple ? 1 : 0;
}

// ------------------------------------------------------------------------------------ key-major
// tau_f: the fp32 thresholds left in `prefix` by emit_kernel.  The tile is computed with the query
// fragment as the row operand and the key fragment as the column operand, so lane l owns key
// (l % 32) and accumulator v is query tile_pos(v) + 4*(l/32) of the tile; the thresholds of a lane's 16
// queries come from a chunk staged in LDS (state rows are padded to whole tiles).
//   WRITE = false: list lengths -> cnt[bh, j];   WRITE = true: lists, starting at col[bh, j].
template <typename T, int R, bool WRITE>
__global__ __launch_bounds__(64) void emit_t_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq, int L,
                                                    HeadTable tab, const float *__restrict__ tau_f,
                                                    const int32_t *__restrict__ jcut,
                                                    const int32_t *__restrict__ tile_flag, int32_t *__restrict__ cnt,
                                                    const int64_t *__restrict__ col, int32_t *__restrict__ idxT)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int j0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * Lq * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const float *tau_b = tau_f + (int64_t)bh * padded_len(Lq);
    const int32_t *jcut_b = jcut + (int64_t)bh * padded_len(Lq);
    const int ntiles = (Lq + 31) >> 5;  // query tiles: the axis this kernel walks
    const int32_t *flag_b = tile_flag + (int64_t)bh * ntiles;
    const int lane = threadIdx.x;
    const int n = lane & 31, half = lane >> 5;
    const bool live = j0 + n < L;
    const int j = min(j0 + n, L - 1);

    const Frag<T, R> kf = load_frag<T, R>(Kb, j0, L, lane);
    __shared__ __align__(16) EmitShared sh;
    if (WRITE && half == 0) {
        // col comes from the counting pass over the same predicate, so the lists fill the head's block of
        // L * k entries exactly; the clamps (to [0, cap], b1 >= b0) only keep an inconsistent col from sending writes out of it
        const int64_t cap = (int64_t)Lq * tab.k[slot];
        const int64_t *cp = col + (int64_t)bh * (L + 1) + j;
        const int64_t b0 = cp[0] < 0 ? 0 : (cp[0] < cap ? cp[0] : cap);
        const int64_t b1 = cp[1] < b0 ? b0 : (cp[1] < cap ? cp[1] : cap);
        sh.out[n] = OwnerOut{tab.off[slot] + b0, 0, live ? (int)(b1 - b0) : 0};
    }
    int wpos = 0;  // WRITE = false: this key's list length
    // Thresholds of the queries, kTauTiles tiles at a time: one coalesced 16-byte load per lane, parked in
    // LDS, from where each lane picks the 16 values of its accumulators with broadcast reads.  (Fetching
    // them per tile straight from memory took four full-width load instructions per tile -- four times
    // the address-path time of the tile's own fragment.)
    constexpr int kTauTiles = 8;
    __shared__ __align__(16) float tau_s[kTauTiles * 32];
    const int npad = padded_len(Lq);
    float4 tau_next = *reinterpret_cast<const float4 *>(tau_b + min(lane * 4, npad - 4));
    Frag<T, R> qf_next = load_frag<T, R>(Qb, 0, Lq, lane);
    for (int qc = 0; qc < ntiles; qc += kTauTiles) {
        *reinterpret_cast<float4 *>(tau_s + lane * 4) = tau_next;
        tau_next = *reinterpret_cast<const float4 *>(tau_b + min((qc + kTauTiles) * 32 + lane * 4, npad - 4));
        const int tn = min(kTauTiles, ntiles - qc);
        for (int t = 0; t < tn; ++t) {
            const int qt = qc + t;
            const int q0 = qt * 32;
            const Frag<T, R> qf = qf_next;
            qf_next = load_frag<T, R>(Qb, q0 + 32, Lq, lane);
            const floatx16_t acc = score_tile<T, R>(qf, kf);
            const uint32_t valid = (q0 + 32 <= Lq) ? 0xFFFFFFFFu : ((1u << (Lq - q0)) - 1u);
            // thresholds of this lane's 16 queries (tile rows 8g + 4*half + 0..3)
            float tq[16];
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const float4 t4 = *reinterpret_cast<const float4 *>(tau_s + t * 32 + 8 * gq + 4 * half);
                tq[4 * gq + 0] = t4.x; tq[4 * gq + 1] = t4.y; tq[4 * gq + 2] = t4.z; tq[4 * gq + 3] = t4.w;
            }
            uint32_t m;
            if (flag_b[qt]) {
                DSV_SIGNMASK16(m, acc[v] - tq[v]);  // score < tau as the sign of (score - tau)
                m = ~m & 0x0F0F0F0Fu;
            } else {
                int jq[16];
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int4 c4 = *reinterpret_cast<const int4 *>(jcut_b + q0 + 8 * gq + 4 * half);
                    jq[4 * gq + 0] = c4.x; jq[4 * gq + 1] = c4.y; jq[4 * gq + 2] = c4.z; jq[4 * gq + 3] = c4.w;
                }
                DSV_MASK16(m, acc[v] > tq[v] || (acc[v] == tq[v] && j <= jq[v]));
            }
            uint32_t sel = merge_halves(m, half) & valid;
            if (!live) sel = 0u;
            if (WRITE) {
                if (half == 0) sh.mask[qt % kBatch][n] = sel;
                if (qt % kBatch == kBatch - 1) expand_batch(sh, idxT, qt - (kBatch - 1), kBatch, lane);
            } else {
                wpos += __popc(sel);
            }
        }
    }
    if (WRITE && ntiles % kBatch) expand_batch(sh, idxT, ntiles - ntiles % kBatch, ntiles % kBatch, lane);
    if (!WRITE && live && half == 0) cnt[(int64_t)bh * L + j] = wpos;
}

// One block per (b, h): exclusive scan of cnt [L] into col [L+1] (int64).
__global__ __launch_bounds__(1024) void list_scan_kernel(const int32_t *__restrict__ cnt, int64_t *__restrict__ col,
                                                         int L)
{
    __shared__ int64_t part[1024];
    const int bh = blockIdx.x;
    const int32_t *c = cnt + (int64_t)bh * L;
    int64_t *o = col + (int64_t)bh * (L + 1);
    const int per = (L + 1023) / 1024;
    const int lo = min((int)threadIdx.x * per, L), hi = min(lo + per, L);
    int64_t sum = 0;
    for (int e = lo; e < hi; ++e) sum += c[e];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int step = 1; step < 1024; step <<= 1) {
        const int64_t add = threadIdx.x >= (unsigned)step ? part[threadIdx.x - step] : 0;
        __syncthreads();
        part[threadIdx.x] += add;
        __syncthreads();
    }
    int64_t run = part[threadIdx.x] - sum;
    for (int e = lo; e < hi; ++e) {
        o[e] = run;
        run += c[e];
    }
    if (threadIdx.x == 1023) o[L] = part[1023];
}

// ------------------------------------------------------------------------------------ host
template <typename T, int R>
static dsv_status emit_all_t(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr,
                             const void *Klr, const SelectBuffers &b, hipStream_t st)
{
    const T *Ql = (const T *)Qlr;
    const T *Kl = (const T *)Klr;
    const int tiles = (p.L + 31) / 32;    // key tiles
    const int qtiles = (Lq + 31) / 32;    // query (or query-group) tiles
    const float *tau_f = reinterpret_cast<const float *>(b.prefix);
    {
        KernelSpan span(DSV_KERNEL_EMIT, st);
        for (int t = 0; t < n_tabs; ++t) {
            dim3 grid(qtiles, tabs[t].n);
            hipLaunchKernelGGL((emit_kernel<T, R>), grid, dim3(64), 0, st, Ql, Kl, Lq, p.L, tabs[t], b.prefix, b.krem, b.idx,
                               b.jcut, b.tile_flag);
            DSV_LAUNCH_CHECK();
        }
    }
    if (b.idx_t) {
        {
            KernelSpan span(DSV_KERNEL_EMIT_T_COUNT, st);
            for (int t = 0; t < n_tabs; ++t) {
                dim3 grid(tiles, tabs[t].n);
                hipLaunchKernelGGL((emit_t_kernel<T, R, false>), grid, dim3(64), 0, st, Ql, Kl, Lq, p.L, tabs[t], tau_f,
                                   b.jcut, b.tile_flag, b.cnt, (const int64_t *)nullptr, (int32_t *)nullptr);
                DSV_LAUNCH_CHECK();
            }
        }
        hipLaunchKernelGGL(list_scan_kernel, dim3(p.B * p.H), dim3(1024), 0, st, b.cnt, b.col, p.L);
        DSV_LAUNCH_CHECK();
        KernelSpan span(DSV_KERNEL_EMIT_T_WRITE, st);
        for (int t = 0; t < n_tabs; ++t) {
            dim3 grid(tiles, tabs[t].n);
            hipLaunchKernelGGL((emit_t_kernel<T, R, true>), grid, dim3(64), 0, st, Ql, Kl, Lq, p.L, tabs[t], tau_f, b.jcut,
                               b.tile_flag, (int32_t *)nullptr, b.col, b.idx_t);
            DSV_LAUNCH_CHECK();
        }
    }
    return DSV_OK;
}

dsv_status launch_emit(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                       const SelectBuffers &b, hipStream_t st)
{
#define DSV_CASE(TT, RR) return emit_all_t<TT, RR>(p, Lq, tabs, n_tabs, Qlr, Klr, b, st)
    if (p.dtype == DSV_BF16) {
        if (p.r == 16) DSV_CASE(bf16_t, 16);
        if (p.r == 32) DSV_CASE(bf16_t, 32);
        if (p.r == 64) DSV_CASE(bf16_t, 64);
    } else if (p.dtype == DSV_F32) {
        if (p.r == 16) DSV_CASE(float, 16);
        if (p.r == 32) DSV_CASE(float, 32);
        if (p.r == 64) DSV_CASE(float, 64);
    }
#undef DSV_CASE
    return DSV_EUNSUPPORTED;
}

}  // namespace dsv
