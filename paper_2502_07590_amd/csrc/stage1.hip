// Stage 1: critical-KV estimation (paper Sec. "Low-Rank based Sparsity Prediction" and
// Sec. "Critical KV Estimation with Kernel Fusion"; two-pass threshold form of Appendix
// "Implementation details").
//
//   project      Q_lr = Q Wq, K_lr = K Wk            (fp32 accumulate, rounded to the storage type)
//   select       per (head, query): exact value of the k-th largest score by a radix search on the
//                order-preserving bit pattern of the fp32 score (four 8-bit digits, one pass over
//                all keys per digit, histograms in LDS), then
//   emit         (stage1_emit.hip) one more pass that writes every key above the threshold plus the
//                lowest-index ties, in ascending key order; optionally the same key-major.
// Scores are recomputed in every pass on the matrix cores (one 32x32 MFMA tile = 32 keys x 32
// queries); the L x L matrix never exists in memory.  Every pass uses the same instruction
// sequence for a score, so a score has the same bits in every pass.
#include <algorithm>
#include <atomic>

#include "stage1_core.h"

namespace dsv {

// ------------------------------------------------------------------------------------ projection
// Q holds Lq rows per head and K holds Lk (equal for per-query selection; with query grouping only the
// groups' centre queries are projected and scored).  One block projects TOK token rows.  X tile and W are staged in LDS as fp32; each thread then
// forms a few outputs of one token with a plain ascending-c fp32 FMA chain.
template <typename T, int D, int R>
__global__ __launch_bounds__(256) void project_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                      const T *__restrict__ Wq, const T *__restrict__ Wk,
                                                      T *__restrict__ Qlr, T *__restrict__ Klr, int Lq, int Lk, int H)
{
    constexpr int TOK = (D * R >= 128 * 64) ? 32 : 64;  // keeps the two tiles under 64 KB of LDS
    constexpr int TPT = 256 / TOK;                       // threads per token
    constexpr int NOUT = R / TPT;                        // outputs per thread
    __shared__ float Xs[TOK][D + 1];
    __shared__ float Ws[D][R];
    const int bh = blockIdx.y;
    const int h = bh % H;
    const int L = blockIdx.z ? Lk : Lq;  // tokens on this side (the grid covers the longer side)
    if ((int)blockIdx.x * TOK >= L) return;
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

// ------------------------------------------------------------------------------------ radix pass
// One digit of the search for the k-th largest score of each query.  Block = 32 queries of one
// head, kRadixWaves waves striding over the key tiles, one shared histogram in LDS laid out [256 digits][32
// queries]: the bank of a counter depends on the query alone, so the 32 lanes of a half-wave (32
// different queries) never collide, whatever their digits are.
//   PASS 0 counts every key by the top digit; PASS p counts only keys whose higher digits equal
//   the prefix found so far.  Afterwards: the digit whose bucket holds the k_rem-th largest
//   remaining key is appended to the prefix and k_rem is reduced by the keys in higher buckets.
// After pass 3 the prefix is the full key of the k-th largest score and |k_rem| is the number of
// keys equal to it that belong to the top-k (at least 1); k_rem < 0 marks "all of them".

// One 32-query tile (queries q0 .. q0+31 of head slot `slot`); hist: the block's 256 x 32 counters.
template <typename T, int R, int PASS>
__device__ __forceinline__ void radix_pass_tile(uint32_t *hist, const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq,
                                                int L, const HeadTable &tab, int slot, int q0, uint32_t *__restrict__ prefix,
                                                int32_t *__restrict__ krem)
{
    constexpr int SHIFT = 24 - 8 * PASS;
    const int bh = tab.bh[slot];
    const T *Qb = Qlr + (int64_t)bh * Lq * R;   // Lq query rows (all L tokens, or one proxy per query group)
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;

    for (int e = threadIdx.x; e < 256 * 32; e += 64 * kRadixWaves) hist[e] = 0;
    __syncthreads();

    const int qi = min(q0 + n, Lq - 1);
    uint32_t pre = 0;
    if constexpr (PASS > 0) pre = prefix[(int64_t)bh * padded_len(Lq) + qi];
    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, Lq, lane);
    const int ntiles = (L + 31) >> 5;
    const int nfull = L >> 5;  // tiles with all 32 keys in range
    uint32_t *hcol_mine = hist + n;  // counter of digit b: hcol_mine[32 * b]
    // When every query of the tile has a threshold prefix in the positive floats (the usual case:
    // k < L/2), a score matches the prefix iff its RAW bits do: negative scores have the sign bit
    // set and can never match, and for positive floats the raw pattern is already monotone.  That
    // drops the key transform from the hot loop: one xor + one compare per score, digits are only
    // extracted for the few matches.
    bool fast = false;
    if constexpr (PASS > 0) fast = __all((pre & 0x80000000u) != 0u);
    if (fast) {
        const uint32_t raw_pre = pre ^ 0x80000000u;
        Frag<T, R> kf_next = load_frag<T, R>(Kb, wave * 32, L, lane);
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            // the next tile's fragment is requested before this tile is scored (rows past the end clamp)
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
            constexpr uint32_t kLimit = 1u << ((SHIFT + 8) & 31);
            if constexpr (PASS >= 2) {
                // Matches are rare from the third digit on (a 16-bit prefix leaves about one score in a
                // thousand): look at four scores at a time with plain xor / min, and only enter the
                // masked histogram update for a group in which some lane has a match.
#pragma unroll
                for (int v0 = 0; v0 < 16; v0 += 4) {
                    uint32_t x[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) x[u] = __float_as_uint(acc[v0 + u]) ^ raw_pre;
                    const uint32_t lo = min(min(x[0], x[1]), min(x[2], x[3]));
                    if (__any(lo < kLimit)) {
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            if (x[u] < kLimit) atomicAdd(&hcol_mine[((x[u] >> SHIFT) & 255u) * 32], 1u);
                    }
                }
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const uint32_t bits = __float_as_uint(acc[v]);
                    if ((bits ^ raw_pre) < kLimit) atomicAdd(&hcol_mine[((bits >> SHIFT) & 255u) * 32], 1u);
                }
            }
        }
    } else {
        Frag<T, R> kf_next = load_frag<T, R>(Kb, wave * 32, L, lane);
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                if constexpr (PASS == 0) {
                    // first digit: counted by the RAW top byte (no key transform in the loop); the scan
                    // below visits the raw buckets in key order
                    atomicAdd(&hcol_mine[(__float_as_uint(acc[v]) >> 24) * 32], 1u);
                } else {
                    const uint32_t key = score_key(acc[v]);
                    if ((key >> (SHIFT + 8)) == (pre >> (SHIFT + 8))) atomicAdd(&hcol_mine[((key >> SHIFT) & 255u) * 32], 1u);
                }
            }
        }
    }
    if (nfull < ntiles && wave == nfull % kRadixWaves) {  // the ragged last tile
        const int j0 = nfull * 32;
        const Frag<T, R> kf = load_frag<T, R>(Kb, j0, L, lane);
        const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t key = score_key(acc[v]);
            bool ok = j0 + tile_pos(v) + 4 * half < L;
            if constexpr (PASS > 0) ok = ok && ((key >> (SHIFT + 8)) == (pre >> (SHIFT + 8)));
            const uint32_t bucket = PASS == 0 ? __float_as_uint(acc[v]) >> 24 : (key >> SHIFT) & 255u;
            if (ok) atomicAdd(&hcol_mine[bucket * 32], 1u);
        }
    }
    __syncthreads();

    if (threadIdx.x < 32 && q0 + (int)threadIdx.x < Lq) {
        const int64_t g = (int64_t)bh * padded_len(Lq) + q0 + threadIdx.x;
        const int kr = PASS == 0 ? tab.k[slot] : krem[g];
        const uint32_t *hcol = hist + threadIdx.x;
        int above = 0, digit = 0;
        // bucket of key digit b: the digit itself, except in pass 0, whose buckets are raw top bytes
        // (positive floats: key digit = raw ^ 0x80; negative floats: key digit = ~raw)
        auto bucket_of = [](int b) { return PASS == 0 ? (b >= 128 ? b ^ 0x80 : b ^ 0xFF) : b; };
        for (int b = 255; b >= 0; --b) {
            const int c = (int)hcol[32 * bucket_of(b)];
            if (above + c >= kr) { digit = b; break; }
            above += c;
        }
        const uint32_t mypre = PASS == 0 ? 0u : prefix[g];
        prefix[g] = mypre | ((uint32_t)digit << SHIFT);
        // after the last digit the bucket holds exactly the keys equal to the threshold: a negative
        // k_rem tells the emission that all of them are taken (then "score >= threshold" decides)
        const int want = kr - above;
        krem[g] = (PASS == 3 && want == (int)hcol[32 * bucket_of(digit)]) ? -want : want;
    }
}

template <typename T, int R, int PASS>
__global__ __launch_bounds__(64 * kRadixWaves) void radix_pass_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq, int L,
                                                         HeadTable tab, uint32_t *__restrict__ prefix,
                                                         int32_t *__restrict__ krem)
{
    __shared__ uint32_t hist[256 * 32];
    radix_pass_tile<T, R, PASS>(hist, Qlr, Klr, Lq, L, tab, blockIdx.y, blockIdx.x * 32, prefix, krem);
}

// The same digit pass for the query tiles on a list (todo[0] = their number, todo[1 + i] = slot * qtiles +
// tile): the tiles the windowed search (stage1_window.hip) could not settle.  The grid is fixed; an empty
// list costs a launch.
template <typename T, int R, int PASS>
__global__ __launch_bounds__(64 * kRadixWaves) void radix_pass_list_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr,
                                                              int Lq, int L, HeadTable tab, uint32_t *__restrict__ prefix,
                                                              int32_t *__restrict__ krem, const int32_t *__restrict__ todo,
                                                              int qtiles)
{
    __shared__ uint32_t hist[256 * 32];
    const int n = min(todo[0], tab.n * qtiles);
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const int id = todo[1 + i];
        const int slot = id / qtiles;
        if (slot >= 0 && slot < tab.n)  // an id outside the table can only come from a corrupted list
            radix_pass_tile<T, R, PASS>(hist, Qlr, Klr, Lq, L, tab, slot, (id - slot * qtiles) * 32, prefix, krem);
        __syncthreads();  // the tile's last readers of hist are done before the next tile clears it
    }
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
static dsv_status project_t(const dsv_problem &p, int Lq, const void *Q, const void *K, const void *Wq, const void *Wk,
                            void *Qlr, void *Klr, hipStream_t st)
{
    constexpr int TOK = (D * R >= 128 * 64) ? 32 : 64;  // must match project_kernel
    dim3 grid((std::max(p.L, Lq) + TOK - 1) / TOK, p.B * p.H, 2);
    hipLaunchKernelGGL((project_kernel<T, D, R>), grid, dim3(256), 0, st, (const T *)Q, (const T *)K, (const T *)Wq,
                       (const T *)Wk, (T *)Qlr, (T *)Klr, Lq, p.L, p.H);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

template <typename T, int D>
static dsv_status project_r(const dsv_problem &p, int Lq, const void *Q, const void *K, const void *Wq, const void *Wk,
                            void *Qlr, void *Klr, hipStream_t st)
{
    switch (p.r) {
    case 16: return project_t<T, D, 16>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
    case 32: return project_t<T, D, 32>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
    case 64: return project_t<T, D, 64>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
    default: return DSV_EUNSUPPORTED;
    }
}

dsv_status launch_project(const dsv_problem &p, int Lq, const void *Q, const void *K, const void *Wq, const void *Wk,
                          void *Qlr, void *Klr, hipStream_t st)
{
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) return project_r<bf16_t, 64>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
        if (p.d == 128) return project_r<bf16_t, 128>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) return project_r<float, 64>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
        if (p.d == 128) return project_r<float, 128>(p, Lq, Q, K, Wq, Wk, Qlr, Klr, st);
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

static std::atomic<int> g_threshold_search{0};
int set_threshold_search(int mode) { return mode < 0 ? g_threshold_search.load() : g_threshold_search.exchange(mode); }

// Which head slots take the windowed search (mode: see set_threshold_search).
static bool slot_takes_window(const dsv_problem &p, int k, int mode)
{
    return mode != 1 && window_sample_keys(p.L, k, mode == 2) > 0;
}

template <typename T, int R>
static dsv_status select_t(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                           const SelectBuffers &b, hipStream_t st)
{
    const T *Ql = (const T *)Qlr;
    const T *Kl = (const T *)Klr;
    const int qtiles = (Lq + 31) / 32;
    const int mode = b.win && b.todo ? g_threshold_search.load() : 1;
    {
        KernelSpan span(DSV_KERNEL_THRESHOLD, st);
        for (int t = 0; t < n_tabs; ++t) {
            HeadTable radix{}, window{};  // the table's slots by search method
            for (int s = 0; s < tabs[t].n; ++s) {
                HeadTable &dst = slot_takes_window(p, tabs[t].k[s], mode) ? window : radix;
                dst.bh[dst.n] = tabs[t].bh[s];
                dst.k[dst.n] = tabs[t].k[s];
                dst.off[dst.n] = tabs[t].off[s];
                ++dst.n;
            }
            const dim3 block(64 * kRadixWaves);
            if (radix.n) {
                dim3 grid(qtiles, radix.n);
                hipLaunchKernelGGL((radix_pass_kernel<T, R, 0>), grid, block, 0, st, Ql, Kl, Lq, p.L, radix, b.prefix, b.krem);
                hipLaunchKernelGGL((radix_pass_kernel<T, R, 1>), grid, block, 0, st, Ql, Kl, Lq, p.L, radix, b.prefix, b.krem);
                hipLaunchKernelGGL((radix_pass_kernel<T, R, 2>), grid, block, 0, st, Ql, Kl, Lq, p.L, radix, b.prefix, b.krem);
                hipLaunchKernelGGL((radix_pass_kernel<T, R, 3>), grid, block, 0, st, Ql, Kl, Lq, p.L, radix, b.prefix, b.krem);
                DSV_LAUNCH_CHECK();
            }
            if (window.n) {
                const dsv_status rc = launch_window_search(p, Lq, window, Qlr, Klr, b, st);
                if (rc != DSV_OK) return rc;
                // the tiles it listed (normally none): the grid is fixed, the blocks walk the list
                const dim3 grid((unsigned)std::min<int64_t>((int64_t)qtiles * window.n, 2048));
                hipLaunchKernelGGL((radix_pass_list_kernel<T, R, 0>), grid, block, 0, st, Ql, Kl, Lq, p.L, window, b.prefix, b.krem, (const int32_t *)b.todo, qtiles);
                hipLaunchKernelGGL((radix_pass_list_kernel<T, R, 1>), grid, block, 0, st, Ql, Kl, Lq, p.L, window, b.prefix, b.krem, (const int32_t *)b.todo, qtiles);
                hipLaunchKernelGGL((radix_pass_list_kernel<T, R, 2>), grid, block, 0, st, Ql, Kl, Lq, p.L, window, b.prefix, b.krem, (const int32_t *)b.todo, qtiles);
                hipLaunchKernelGGL((radix_pass_list_kernel<T, R, 3>), grid, block, 0, st, Ql, Kl, Lq, p.L, window, b.prefix, b.krem, (const int32_t *)b.todo, qtiles);
                DSV_LAUNCH_CHECK();
            }
        }
    }
    return launch_emit(p, Lq, tabs, n_tabs, Qlr, Klr, b, st);
}

dsv_status launch_select(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                         const SelectBuffers &b, hipStream_t st)
{
#define DSV_CASE(TT, RR) return select_t<TT, RR>(p, Lq, tabs, n_tabs, Qlr, Klr, b, st)
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
