// Stage 1: critical-KV estimation (paper Sec. "Low-Rank based Sparsity Prediction" and
// Sec. "Critical KV Estimation with Kernel Fusion"; two-pass threshold form of Appendix
// "Implementation details").
//
//   project      Q_lr = Q Wq, K_lr = K Wk            (fp32 accumulate, rounded to the storage type)
//   select       per (head, query): exact value of the k-th largest score by a radix search on the
//                order-preserving bit pattern of the fp32 score (four 8-bit digits, one pass over
//                all keys per digit, histograms in LDS), then
//   emit         one more pass that writes every key above the threshold plus the lowest-index
//                ties, in ascending key order.
// Scores are recomputed in every pass on the matrix cores (one 32x32 MFMA tile = 32 keys x 32
// queries); the L x L matrix never exists in memory.  Every pass uses the same instruction
// sequence for a score, so a score has the same bits in every pass.
#include "common.h"

namespace dsv {

// ------------------------------------------------------------------------------------ projection
// One block projects TOK token rows.  X tile and W are staged in LDS as fp32; each thread then
// forms a few outputs of one token with a plain ascending-c fp32 FMA chain.
template <typename T, int D, int R>
__global__ __launch_bounds__(256) void project_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                      const T *__restrict__ Wq, const T *__restrict__ Wk,
                                                      T *__restrict__ Qlr, T *__restrict__ Klr, int L, int H)
{
    constexpr int TOK = (D * R >= 128 * 64) ? 32 : 64;  // keeps the two tiles under 64 KB of LDS
    constexpr int TPT = 256 / TOK;                       // threads per token
    constexpr int NOUT = R / TPT;                        // outputs per thread
    __shared__ float Xs[TOK][D + 1];
    __shared__ float Ws[D][R];
    const int bh = blockIdx.y;
    const int h = bh % H;
    const T *X = (blockIdx.z ? K : Q) + (int64_t)bh * L * D;
    const T *W = (blockIdx.z ? Wk : Wq) + (int64_t)h * D * R;
    T *out = (blockIdx.z ? Klr : Qlr) + (int64_t)bh * L * R;
    const int t0 = blockIdx.x * TOK;
    const int ntok = min(TOK, L - t0);

    for (int e = threadIdx.x; e < D * R; e += 256) Ws[e / R][e % R] = to_f32<T>(W[e]);
    for (int e = threadIdx.x; e < TOK * D; e += 256) {
        int tok = e / D, c = e % D;
        Xs[tok][c] = tok < ntok ? to_f32<T>(X[(int64_t)(t0 + tok) * D + c]) : 0.f;
    }
    __syncthreads();

    const int tok = threadIdx.x / TPT;
    const int tbase = (threadIdx.x % TPT) * NOUT;
    float acc[NOUT];
#pragma unroll
    for (int t = 0; t < NOUT; ++t) acc[t] = 0.f;
    for (int c = 0; c < D; ++c) {
        float x = Xs[tok][c];
#pragma unroll
        for (int t = 0; t < NOUT; ++t) acc[t] = fmaf(x, Ws[c][tbase + t], acc[t]);
    }
    if (tok < ntok) {
#pragma unroll
        for (int t = 0; t < NOUT; ++t) out[(int64_t)(t0 + tok) * R + tbase + t] = from_f32<T>(acc[t]);
    }
}

// ------------------------------------------------------------------------------------ score tiles
// MFMA operand fragment of 32 rows of a [*, R] low-rank matrix.  Lane l holds row (l % 32) and the
// K-slice selected by (l / 32); keys go in as the A operand, queries as the B operand, so that
// acc[v] of lane l is the score of query (l % 32) against key 8*(v/4) + 4*(l/32) + (v%4) of the tile.
template <typename T, int R> struct Frag;
template <int R> struct Frag<bf16_t, R> { bf16x8_t v[R / 16]; };
template <int R> struct Frag<float, R> { float v[R / 2]; };

template <typename T, int R>
__device__ __forceinline__ Frag<T, R> load_frag_row(const T *__restrict__ base, int64_t row, int lane)
{
    Frag<T, R> f;
    const int half = lane >> 5;
    const T *p = base + row * R;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int m = 0; m < R / 16; ++m) f.v[m] = *reinterpret_cast<const bf16x8_t *>(p + m * 16 + half * 8);
    } else {
#pragma unroll
        for (int m = 0; m < R / 2; ++m) f.v[m] = p[2 * m + half];
    }
    return f;
}

// Rows row0 .. row0+31 of the matrix; rows past the end are clamped (callers mask their results).
template <typename T, int R>
__device__ __forceinline__ Frag<T, R> load_frag(const T *__restrict__ base, int row0, int L, int lane)
{
    return load_frag_row<T, R>(base, min(row0 + (lane & 31), L - 1), lane);
}

template <typename T, int R>
__device__ __forceinline__ floatx16_t score_tile(const Frag<T, R> &keys, const Frag<T, R> &queries)
{
    floatx16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int m = 0; m < R / 16; ++m)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(keys.v[m], queries.v[m], acc, 0, 0, 0);
    } else {
#pragma unroll
        for (int m = 0; m < R / 2; ++m)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(keys.v[m], queries.v[m], acc, 0, 0, 0);
    }
    return acc;
}

// Position inside a 32-key tile of accumulator v for a lane in half 0 (half 1 adds 4).
__device__ __forceinline__ constexpr int tile_pos(int v) { return 8 * (v / 4) + (v % 4); }

// Order-preserving map fp32 -> uint32 (larger float <=> larger key), and its inverse.
__device__ __forceinline__ uint32_t score_key(float s)
{
    uint32_t u = __float_as_uint(s);
    return u ^ ((uint32_t)((int32_t)u >> 31) | 0x80000000u);
}
__device__ __forceinline__ float key_score(uint32_t key)
{
    return __uint_as_float((key & 0x80000000u) ? (key ^ 0x80000000u) : ~key);
}

// ------------------------------------------------------------------------------------ radix pass
// One digit of the search for the k-th largest score of each query.  Block = 32 queries of one
// head, 4 waves striding over the key tiles, one shared [32][256] histogram in LDS (row stride 257
// words so that equal digits of different queries fall in different banks).
//   PASS 0 counts every key by the top digit; PASS p counts only keys whose higher digits equal
//   the prefix found so far.  Afterwards: the digit whose bucket holds the k_rem-th largest
//   remaining key is appended to the prefix and k_rem is reduced by the keys in higher buckets.
// After pass 3 the prefix is the full key of the k-th largest score and k_rem is the number of
// keys equal to it that belong to the top-k (at least 1).
template <typename T, int R, int PASS>
__global__ __launch_bounds__(256) void radix_pass_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int L,
                                                         HeadTable tab, uint32_t *__restrict__ prefix,
                                                         int32_t *__restrict__ krem)
{
    constexpr int STRIDE = 257;
    constexpr int SHIFT = 24 - 8 * PASS;
    __shared__ uint32_t hist[32 * STRIDE];
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * L * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;

    for (int e = threadIdx.x; e < 32 * STRIDE; e += 256) hist[e] = 0;
    __syncthreads();

    const int qi = min(q0 + n, L - 1);
    uint32_t pre = 0;
    if constexpr (PASS > 0) pre = prefix[(int64_t)bh * L + qi];
    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, L, lane);
    const int ntiles = (L + 31) >> 5;
    for (int tile = wave; tile < ntiles; tile += 4) {
        const int j0 = tile * 32;
        const Frag<T, R> kf = load_frag<T, R>(Kb, j0, L, lane);
        const floatx16_t acc = score_tile<T, R>(kf, qf);
        const bool full = j0 + 32 <= L;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t key = score_key(acc[v]);
            bool ok = full || (j0 + tile_pos(v) + 4 * half < L);
            if constexpr (PASS > 0) ok = ok && ((key >> (SHIFT + 8)) == (pre >> (SHIFT + 8)));
            if (ok) atomicAdd(&hist[n * STRIDE + ((key >> SHIFT) & 255u)], 1u);
        }
    }
    __syncthreads();

    if (threadIdx.x < 32 && q0 + (int)threadIdx.x < L) {
        const int64_t g = (int64_t)bh * L + q0 + threadIdx.x;
        const int kr = PASS == 0 ? tab.k[slot] : krem[g];
        const uint32_t *hrow = hist + threadIdx.x * STRIDE;
        int above = 0, digit = 0;
        for (int b = 255; b >= 0; --b) {
            const int c = (int)hrow[b];
            if (above + c >= kr) { digit = b; break; }
            above += c;
        }
        const uint32_t mypre = PASS == 0 ? 0u : prefix[g];
        prefix[g] = mypre | ((uint32_t)digit << SHIFT);
        krem[g] = kr - above;
    }
}

// ------------------------------------------------------------------------------------ emit
// One wave owns 32 queries of one head and walks the key tiles in ascending order.  A key is
// selected when its score is above the query's threshold, or equal to it while fewer than k_rem
// equal keys have been taken (lowest index first).  Lanes l and l+32 (same query) merge their 16
// predicate bits into one 32-bit mask in key order; each lane then writes its own selected keys at
// cursor + rank, so every row comes out in ascending key index.  jcut[query] receives the index of
// the last tie taken (the k-th key itself is one, so there always is one), so that
//   selected(i, j)  <=>  s_ij > tau_i  or  (s_ij == tau_i and j <= jcut_i)
// is a pure function of the pair, which the key-major emission below re-evaluates.
template <typename T, int R>
__global__ __launch_bounds__(64) void emit_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int L,
                                                  HeadTable tab, const uint32_t *__restrict__ prefix,
                                                  const int32_t *__restrict__ krem, int32_t *__restrict__ idx,
                                                  int32_t *__restrict__ jcut)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * L * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x;
    const int n = lane & 31, half = lane >> 5;
    const bool live = q0 + n < L;
    const int qi = min(q0 + n, L - 1);
    const float tau = key_score(prefix[(int64_t)bh * L + qi]);
    const int ties_wanted = krem[(int64_t)bh * L + qi];
    int32_t *row = idx + tab.off[slot] + (int64_t)qi * k;

    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, L, lane);
    const uint32_t mine_pos = 0x0F0F0F0Fu << (4 * half);
    int cursor = 0, ties_taken = 0, last_tie = -1;
    const int ntiles = (L + 31) >> 5;
    for (int tile = 0; tile < ntiles; ++tile) {
        const int j0 = tile * 32;
        const Frag<T, R> kf = load_frag<T, R>(Kb, j0, L, lane);
        const floatx16_t acc = score_tile<T, R>(kf, qf);
        uint32_t mgt = 0, meq = 0;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            mgt |= (uint32_t)(acc[v] > tau) << tile_pos(v);
            meq |= (uint32_t)(acc[v] == tau) << tile_pos(v);
        }
        mgt <<= 4 * half;
        meq <<= 4 * half;
        mgt |= (uint32_t)__shfl_xor((int)mgt, 32);
        meq |= (uint32_t)__shfl_xor((int)meq, 32);
        const uint32_t valid = (j0 + 32 <= L) ? 0xFFFFFFFFu : ((1u << (L - j0)) - 1u);
        mgt &= valid;
        meq &= valid;
        if (meq) {
            const int room = ties_wanted - ties_taken;
            while (__popc(meq) > room) meq &= ~(0x80000000u >> __clz(meq));  // drop the highest index
            ties_taken += __popc(meq);
            if (meq) last_tie = j0 + 31 - __clz(meq);
        }
        const uint32_t sel = mgt | meq;
        uint32_t mine = sel & mine_pos;
        while (mine) {
            const int pos = __ffs(mine) - 1;
            const int w = cursor + __popc(sel & ((1u << pos) - 1u));
            if (live && w < k) row[w] = j0 + pos;
            mine &= mine - 1;
        }
        cursor += __popc(sel);
    }
    if (jcut && live && half == 0) jcut[(int64_t)bh * L + qi] = last_tie;
}

// ------------------------------------------------------------------------------------ key-major emit
// The transposed index: for every key j, the ascending list of queries that selected it.  One wave
// owns 32 keys of one head and walks the QUERY tiles in ascending order, recomputing each 32x32
// tile with the same operand roles as every other pass (identical score bits) and re-evaluating
// selected(i, j) from tau_i and jcut_i.  For accumulator v the wave-wide ballot is, in its low half,
// the query mask of key tile_pos(v) and, in its high half, that of key tile_pos(v)+4.
//   WRITE = false: count list lengths  -> cnt[bh, j]
//   WRITE = true : lists start at col[bh, j] (exclusive scan of the counts); lanes with a set bit
//                  write their query index at position + rank.
template <typename T, int R, bool WRITE>
__global__ __launch_bounds__(64) void emit_t_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int L,
                                                    HeadTable tab, const uint32_t *__restrict__ prefix,
                                                    const int32_t *__restrict__ jcut, int32_t *__restrict__ cnt,
                                                    const int64_t *__restrict__ col, int32_t *__restrict__ idxT)
{
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int j0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * L * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const uint32_t *pre_b = prefix + (int64_t)bh * L;
    const int32_t *jcut_b = jcut + (int64_t)bh * L;
    const int lane = threadIdx.x;
    const int n = lane & 31, half = lane >> 5;
    const uint32_t below = (1u << n) - 1u;  // lanes of my half with a lower query index

    const Frag<T, R> kf = load_frag<T, R>(Kb, j0, L, lane);
    int32_t *out = WRITE ? idxT + tab.off[slot] : nullptr;
    int64_t pos[16];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int j = j0 + tile_pos(v) + 4 * half;
        pos[v] = (WRITE && j < L) ? col[(int64_t)bh * (L + 1) + j] : 0;
    }
    const int ntiles = (L + 31) >> 5;
    for (int qt = 0; qt < ntiles; ++qt) {
        const int q0 = qt * 32;
        const bool live = q0 + n < L;
        const int qi = min(q0 + n, L - 1);
        const Frag<T, R> qf = load_frag<T, R>(Qb, q0, L, lane);
        const float tau = key_score(pre_b[qi]);
        const int jc = jcut_b[qi];
        const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = j0 + tile_pos(v) + 4 * half;
            const bool pred = live && j < L && (acc[v] > tau || (acc[v] == tau && j <= jc));
            const uint64_t m = __ballot(pred);
            const uint32_t mh = half ? (uint32_t)(m >> 32) : (uint32_t)m;
            if (WRITE) {
                if (pred) out[pos[v] + __popc(mh & below)] = q0 + n;
            }
            pos[v] += __popc(mh);
        }
    }
    if (!WRITE && n == 0) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = j0 + tile_pos(v) + 4 * half;
            if (j < L) cnt[(int64_t)bh * L + j] = (int32_t)pos[v];
        }
    }
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
    for (int j = lo; j < hi; ++j) sum += c[j];
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int step = 1; step < 1024; step <<= 1) {
        const int64_t add = threadIdx.x >= (unsigned)step ? part[threadIdx.x - step] : 0;
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

// ------------------------------------------------------------------------------------ debug scores
// fp32 scores of chosen query rows against every key, through the same tile routine.
template <typename T, int R>
__global__ __launch_bounds__(64) void scores_rows_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int L,
                                                         const int32_t *__restrict__ rows, int n_rows,
                                                         float *__restrict__ scores)
{
    const int lane = threadIdx.x;
    const int n = lane & 31, half = lane >> 5;
    const int r0 = blockIdx.y * 32;
    const int rsel = min(r0 + n, n_rows - 1);
    const Frag<T, R> qf = load_frag_row<T, R>(Qlr, rows[rsel], lane);
    const int j0 = blockIdx.x * 32;
    const Frag<T, R> kf = load_frag<T, R>(Klr, j0, L, lane);
    const floatx16_t acc = score_tile<T, R>(kf, qf);
    if (r0 + n < n_rows) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int j = j0 + tile_pos(v) + 4 * half;
            if (j < L) scores[(int64_t)(r0 + n) * L + j] = acc[v];
        }
    }
}

// ------------------------------------------------------------------------------------ host
template <typename T, int D, int R>
static dsv_status project_t(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                            void *Qlr, void *Klr, hipStream_t st)
{
    constexpr int TOK = (D * R >= 128 * 64) ? 32 : 64;  // must match project_kernel
    dim3 grid((p.L + TOK - 1) / TOK, p.B * p.H, 2);
    hipLaunchKernelGGL((project_kernel<T, D, R>), grid, dim3(256), 0, st, (const T *)Q, (const T *)K, (const T *)Wq,
                       (const T *)Wk, (T *)Qlr, (T *)Klr, p.L, p.H);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status project_r(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                            void *Qlr, void *Klr, hipStream_t st)
{
    switch (p.r) {
    case 16: return project_t<T, D, 16>(p, Q, K, Wq, Wk, Qlr, Klr, st);
    case 32: return project_t<T, D, 32>(p, Q, K, Wq, Wk, Qlr, Klr, st);
    case 64: return project_t<T, D, 64>(p, Q, K, Wq, Wk, Qlr, Klr, st);
    default: return DSV_EUNSUPPORTED;
    }
}

dsv_status launch_project(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                          void *Qlr, void *Klr, hipStream_t st)
{
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) return project_r<bf16_t, 64>(p, Q, K, Wq, Wk, Qlr, Klr, st);
        if (p.d == 128) return project_r<bf16_t, 128>(p, Q, K, Wq, Wk, Qlr, Klr, st);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) return project_r<float, 64>(p, Q, K, Wq, Wk, Qlr, Klr, st);
        if (p.d == 128) return project_r<float, 128>(p, Q, K, Wq, Wk, Qlr, Klr, st);
    }
    return DSV_EUNSUPPORTED;
}

template <typename T, int R>
static dsv_status scores_rows_t(const dsv_problem &p, const void *Qlr, const void *Klr, int bh, const int32_t *rows,
                                int n_rows, float *scores, hipStream_t st)
{
    const T *Qb = (const T *)Qlr + (int64_t)bh * p.L * R;
    const T *Kb = (const T *)Klr + (int64_t)bh * p.L * R;
    dim3 grid((p.L + 31) / 32, (n_rows + 31) / 32);
    hipLaunchKernelGGL((scores_rows_kernel<T, R>), grid, dim3(64), 0, st, Qb, Kb, p.L, rows, n_rows, scores);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_scores_rows(const dsv_problem &p, const void *Qlr, const void *Klr, int bh, const int32_t *rows,
                              int n_rows, float *scores, hipStream_t st)
{
#define DSV_CASE(TT, RR) return scores_rows_t<TT, RR>(p, Qlr, Klr, bh, rows, n_rows, scores, st)
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

template <typename T, int R>
static dsv_status select_t(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                           const SelectBuffers &b, hipStream_t st)
{
    const T *Ql = (const T *)Qlr;
    const T *Kl = (const T *)Klr;
    const int qtiles = (p.L + 31) / 32;
    for (int t = 0; t < n_tabs; ++t) {
        dim3 grid(qtiles, tabs[t].n);
        hipLaunchKernelGGL((radix_pass_kernel<T, R, 0>), grid, dim3(256), 0, st, Ql, Kl, p.L, tabs[t], b.prefix, b.krem);
        hipLaunchKernelGGL((radix_pass_kernel<T, R, 1>), grid, dim3(256), 0, st, Ql, Kl, p.L, tabs[t], b.prefix, b.krem);
        hipLaunchKernelGGL((radix_pass_kernel<T, R, 2>), grid, dim3(256), 0, st, Ql, Kl, p.L, tabs[t], b.prefix, b.krem);
        hipLaunchKernelGGL((radix_pass_kernel<T, R, 3>), grid, dim3(256), 0, st, Ql, Kl, p.L, tabs[t], b.prefix, b.krem);
        hipLaunchKernelGGL((emit_kernel<T, R>), grid, dim3(64), 0, st, Ql, Kl, p.L, tabs[t], b.prefix, b.krem, b.idx,
                           b.jcut);
        DSV_LAUNCH_CHECK();
        if (b.idx_t) {
            hipLaunchKernelGGL((emit_t_kernel<T, R, false>), grid, dim3(64), 0, st, Ql, Kl, p.L, tabs[t], b.prefix,
                               b.jcut, b.cnt, (const int64_t *)nullptr, (int32_t *)nullptr);
            DSV_LAUNCH_CHECK();
        }
    }
    if (b.idx_t) {
        hipLaunchKernelGGL(list_scan_kernel, dim3(p.B * p.H), dim3(1024), 0, st, b.cnt, b.col, p.L);
        DSV_LAUNCH_CHECK();
        for (int t = 0; t < n_tabs; ++t) {
            dim3 grid(qtiles, tabs[t].n);
            hipLaunchKernelGGL((emit_t_kernel<T, R, true>), grid, dim3(64), 0, st, Ql, Kl, p.L, tabs[t], b.prefix,
                               b.jcut, (int32_t *)nullptr, b.col, b.idx_t);
            DSV_LAUNCH_CHECK();
        }
    }
    return DSV_OK;
}

dsv_status launch_select(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                         const SelectBuffers &b, hipStream_t st)
{
#define DSV_CASE(TT, RR) return select_t<TT, RR>(p, tabs, n_tabs, Qlr, Klr, b, st)
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
