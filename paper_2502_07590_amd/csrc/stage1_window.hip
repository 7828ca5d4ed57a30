// Stage 1, threshold search in two sweeps over the keys instead of four (paper Sec. "Critical KV
// Estimation with Kernel Fusion": the top-k threshold of every query; Appendix "Implementation details").
//
// The radix search of stage1.hip resolves the 32 bits of the k-th largest score 8 bits per sweep.  Here
// a sample of the keys first brackets that score for every query:
//   sample   scores of a few thousand evenly spaced keys; two order statistics of the sample, a few standard
//            deviations of the sampling error to either side of rank k * (sample / L), resolved to their
//            top 16 bits: [lo, hi] in the order-preserving key space;
//   window   one sweep over all keys: 255 equal bins from lo upward (bin width a power of two, chosen so
//            that they reach past hi) plus one bin for everything above; the bin that holds the k-th
//            largest score follows, as in a radix pass, together with the rank inside it;
//   collect  one sweep that parks the few scores of that bin (a few dozen) in LDS and picks the wanted one
//            exactly, with its number of ties.
// Nothing here is approximate: the sample only decides where the bins lie.  A query whose k-th largest
// score is outside its bracket, or whose bin holds more scores than the LDS slots, puts its tile on a list,
// and the radix search runs on the listed tiles afterwards (stage1.hip, radix_pass_list_kernel) -- with
// uniformly drawn samples that is about one query in 10^8; inputs with massive ties end up there.
// Outputs are those of the radix search: prefix = key of the threshold score, krem = +-(ties to take).
#include <algorithm>
#include <cmath>

#include "stage1_core.h"

namespace dsv {

constexpr int kMinSampleKeys = 2048;  // smallest key sample (64 tiles)
constexpr int kWindowCap = 256;       // scores of the chosen bin that fit the LDS slots of a query

// Per head slot: the sample (tiles of 32 keys; sample key i is row i * stride + stride / 2) and the ranks
// (1 = largest) of its two order statistics: hi bounds the threshold from above, lo from below.
struct WindowRanks {
    int32_t hi[kMaxSlots], lo[kMaxSlots];
    int32_t tiles[kMaxSlots], stride[kMaxSlots];
};

// Rank of the threshold in a sample of n keys and six standard deviations of its sampling error either way.
static void sample_ranks(int L, int k, int n, int &hi, int &lo)
{
    const double frac = (double)k / (double)L;
    const double ks = frac * n;
    const double m = 6.0 * std::sqrt(std::max(ks * (1.0 - frac), 0.0)) + 2.0;
    hi = (int)std::floor(ks - m);
    lo = (int)std::ceil(ks + m);
}

// Keys to sample for a head that keeps k of L keys; 0: the windowed search does not fit that head.
// The sample must be large enough that (a) both order statistics exist in it -- about 64 sample keys above
// the threshold -- and (b) the bracket, whose width in ranks shrinks with the square root of the sample,
// leaves a few dozen scores per bin; and small enough to stay a minor part of the work.  Unless forced,
// the search is also left to the radix passes where it would not pay: short sequences, and thresholds near
// zero (k > L/4), where the float keys spread a narrow band of values over most of the key space.
int window_sample_keys(int L, int k, bool forced)
{
    if (L < 2 * kMinSampleKeys || k < 1 || k >= L) return 0;
    if (!forced && (L < 16384 || (int64_t)k * 4 > L)) return 0;
    const double frac = (double)k / (double)L;
    const double per_bin = (double)L * std::sqrt(frac * (1.0 - frac)) / 700.0;
    const double want = std::max({(double)kMinSampleKeys, 64.0 / frac, per_bin * per_bin});
    const int cap = (forced ? L / 2 : std::min(L / 8, 16384)) / 32 * 32;
    const int n = (int)std::min((double)cap, std::ceil(want / 32.0) * 32.0);
    if (n < kMinSampleKeys) return 0;
    int hi, lo;
    sample_ranks(L, k, n, hi, lo);
    return hi >= 1 && lo <= n ? n : 0;
}

// ------------------------------------------------------------------------------------ sample
template <typename T, int R>
__global__ __launch_bounds__(64 * kRadixWaves) void window_sample_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq, int L,
                                                            HeadTable tab, WindowRanks wr, uint32_t *__restrict__ lo_out,
                                                            uint32_t *__restrict__ hi_out, int32_t *__restrict__ todo)
{
    __shared__ uint32_t hA[256 * 32], hB[256 * 32];  // [digit][query]
    __shared__ int32_t dig[2][32], abv[2][32];
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * Lq * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) todo[0] = 0;  // the list of unsettled tiles starts empty
    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, Lq, lane);
    const int rank[2] = {wr.hi[slot], wr.lo[slot]};
    const int kTiles = wr.tiles[slot], stride = wr.stride[slot];
    const int n_keys = kTiles * 32;

    for (int e = threadIdx.x; e < 256 * 32; e += 64 * kRadixWaves) hA[e] = 0;
    __syncthreads();
    for (int tile = wave; tile < kTiles; tile += kRadixWaves) {
        const int64_t row = (int64_t)(tile * 32 + n) * stride + stride / 2;
        const floatx16_t acc = score_tile<T, R>(load_frag_row<T, R>(Kb, row, lane), qf);
#pragma unroll
        for (int v = 0; v < 16; ++v) atomicAdd(&hA[(score_key(acc[v]) >> 24) * 32 + n], 1u);
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const int q = threadIdx.x & 31, w = threadIdx.x >> 5;
        int d = -1, above = 0;
        if (rank[w] >= 1 && rank[w] <= n_keys) {
            for (int b = 255; b >= 0; --b) {
                const int c = (int)hA[b * 32 + q];
                if (above + c >= rank[w]) { d = b; break; }
                above += c;
            }
        }
        dig[w][q] = d;
        abv[w][q] = above;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 256 * 32; e += 64 * kRadixWaves) { hA[e] = 0; hB[e] = 0; }
    __syncthreads();
    const uint32_t d_hi = (uint32_t)dig[0][n], d_lo = (uint32_t)dig[1][n];  // -1 matches no top byte
    for (int tile = wave; tile < kTiles; tile += kRadixWaves) {
        const int64_t row = (int64_t)(tile * 32 + n) * stride + stride / 2;
        const floatx16_t acc = score_tile<T, R>(load_frag_row<T, R>(Kb, row, lane), qf);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t key = score_key(acc[v]);
            if ((key >> 24) == d_hi) atomicAdd(&hA[((key >> 16) & 255u) * 32 + n], 1u);
            if ((key >> 24) == d_lo) atomicAdd(&hB[((key >> 16) & 255u) * 32 + n], 1u);
        }
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const int q = threadIdx.x & 31, w = threadIdx.x >> 5;
        const int d0 = dig[w][q];
        uint32_t out = w ? 0u : 0xFFFFFFFFu;  // no bound on this side
        if (d0 >= 0) {
            const uint32_t *h = w ? hB : hA;
            const int rem = rank[w] - abv[w][q];
            int above = 0, d1 = 0;
            for (int b = 255; b >= 0; --b) {
                const int c = (int)h[b * 32 + q];
                if (above + c >= rem) { d1 = b; break; }
                above += c;
            }
            const uint32_t key16 = ((uint32_t)d0 << 8) | (uint32_t)d1;
            out = w ? (key16 << 16) : ((key16 << 16) | 0xFFFFu);  // rounded outward
        }
        if (q0 + q < Lq) (w ? lo_out : hi_out)[(int64_t)bh * padded_len(Lq) + q0 + q] = out;
    }
}

// ------------------------------------------------------------------------------------ window
// prefix: lo on entry; on exit the first key of the chosen bin (or the threshold key itself when the bins
// are one key wide).  win: hi on entry; on exit the width of the chosen bin, 0 when the query is settled
// or given up.  krem: rank of the threshold inside the bin (or the final tie count when settled).
template <typename T, int R>
__global__ __launch_bounds__(64 * kRadixWaves) void window_hist_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr, int Lq,
                                                                      int L, HeadTable tab, uint32_t *__restrict__ prefix,
                                                                      uint32_t *__restrict__ win, int32_t *__restrict__ krem,
                                                                      int32_t *__restrict__ todo, int qtiles)
{
    __shared__ uint32_t hist[256 * 32];
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * Lq * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;

    for (int e = threadIdx.x; e < 256 * 32; e += 64 * kRadixWaves) hist[e] = 0;
    __syncthreads();

    const int qi = min(q0 + n, Lq - 1);
    const int64_t g = (int64_t)bh * padded_len(Lq) + qi;
    const uint32_t lo = prefix[g], hi = win[g];
    const uint32_t span = hi >= lo ? hi - lo : 0u;
    // 255 bins of 2^s keys from lo upward reach past hi; bin 255 takes everything above them
    int s = span < 255u ? 0 : 32 - __clz(span) - 8;
    if ((span >> s) >= 255u) ++s;
    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, Lq, lane);
    const int ntiles = (L + 31) >> 5;
    const int nfull = L >> 5;
    uint32_t *hcol_mine = hist + n;
    // every lo a positive float: a score is at or above lo iff its raw bits are, as signed integers
    // (negative scores are negative integers), and its distance from lo is the difference of the raw bits
    const bool fast = __all((lo & 0x80000000u) != 0u);
    Frag<T, R> kf_next = load_frag<T, R>(Kb, wave * 32, L, lane);
    if (fast) {
        const int32_t raw_lo = (int32_t)(lo ^ 0x80000000u);
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t bits = (int32_t)__float_as_uint(acc[v]);
                // some lane of the wave nearly always has a hit: keep the update on the straight path
                if (__builtin_expect(bits >= raw_lo, 1)) atomicAdd(&hcol_mine[min((uint32_t)(bits - raw_lo) >> s, 255u) * 32], 1u);
            }
        }
    } else {
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t key = score_key(acc[v]);
                if (key >= lo) atomicAdd(&hcol_mine[min((key - lo) >> s, 255u) * 32], 1u);
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
            if (j0 + tile_pos(v) + 4 * half < L && key >= lo) atomicAdd(&hcol_mine[min((key - lo) >> s, 255u) * 32], 1u);
        }
    }
    __syncthreads();

    if (threadIdx.x < 32) {  // lane t of wave 0 holds lo and s of query q0 + t
        bool fail = false;
        if (q0 + (int)threadIdx.x < Lq) {
            const int kr = tab.k[slot];
            const uint32_t *hcol = hist + threadIdx.x;
            int cum = (int)hcol[32 * 255], b = -1, cnt = 0;
            if (cum < kr) {
                for (int bb = 254; bb >= 0; --bb) {
                    const int c = (int)hcol[32 * bb];
                    if (cum + c >= kr) { b = bb; cnt = c; break; }
                    cum += c;
                }
            }
            if (b < 0) {
                fail = true;  // the k-th largest score lies above the bins or below lo
            } else {
                const int want = kr - cum;
                prefix[g] = lo + ((uint32_t)b << s);
                if (s == 0) {  // the bin is a single score value: settled
                    krem[g] = want == cnt ? -want : want;
                    win[g] = 0u;
                } else if (cnt > kWindowCap) {
                    fail = true;
                } else {
                    krem[g] = want;
                    win[g] = 1u << s;
                }
            }
            if (fail) win[g] = 0u;
        }
        if (__any(fail) && threadIdx.x == 0) {
            const int at = atomicAdd(&todo[0], 1);
            if (at >= 0 && at < tab.n * qtiles) todo[1 + at] = slot * qtiles + blockIdx.x;
        }
    }
}

// ------------------------------------------------------------------------------------ collect
template <typename T, int R>
__global__ __launch_bounds__(64 * kRadixWaves) void window_collect_kernel(const T *__restrict__ Qlr, const T *__restrict__ Klr,
                                                                         int Lq, int L, HeadTable tab,
                                                                         uint32_t *__restrict__ prefix,
                                                                         const uint32_t *__restrict__ win,
                                                                         int32_t *__restrict__ krem)
{
    constexpr int TPQ = 64 * kRadixWaves / 32;         // threads per query in the final selection
    __shared__ uint32_t cand[32][kWindowCap + 1];      // padded: the selection reads one column per query
    __shared__ int32_t ccnt[32];
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int q0 = blockIdx.x * 32;
    const T *Qb = Qlr + (int64_t)bh * Lq * R;
    const T *Kb = Klr + (int64_t)bh * L * R;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;
    const int64_t g0 = (int64_t)bh * padded_len(Lq) + q0;
    const bool live = q0 + n < Lq;
    const uint32_t base = live ? prefix[g0 + n] : 0u;
    const uint32_t width = live ? win[g0 + n] : 0u;   // 0: nothing to collect for this query
    if (__all(width == 0u)) return;                    // same 32 queries in every wave: the whole block leaves
    if (threadIdx.x < 32) ccnt[threadIdx.x] = 0;
    __syncthreads();

    const Frag<T, R> qf = load_frag<T, R>(Qb, q0, Lq, lane);
    const int ntiles = (L + 31) >> 5;
    const int nfull = L >> 5;
    auto park = [&](uint32_t key) {
        const int at = atomicAdd(&ccnt[n], 1);
        if (at < kWindowCap) cand[n][at] = key;
    };
    // Bins of positive floats well below the top of the exponent range: distance from the bin's first key
    // = difference of the raw bits, and the raw bits of a negative score (>= 2^31) are at least 3 * 2^24
    // away from any such raw base, above every bin width (<= 2^25).
    const bool fast = __all(width == 0u || ((base & 0x80000000u) != 0u && (base ^ 0x80000000u) <= 0x7D000000u));
    Frag<T, R> kf_next = load_frag<T, R>(Kb, wave * 32, L, lane);
    if (fast) {
        const uint32_t raw_base = base ^ 0x80000000u;
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
            for (int v0 = 0; v0 < 16; v0 += 4) {  // hits are rare: look at four scores at a time
                uint32_t x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) x[u] = __float_as_uint(acc[v0 + u]) - raw_base;
                const uint32_t lo4 = min(min(x[0], x[1]), min(x[2], x[3]));
                if (__any(lo4 < width)) {
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        if (x[u] < width) park(base + x[u]);
                }
            }
        }
    } else {
        for (int tile = wave; tile < nfull; tile += kRadixWaves) {
            const Frag<T, R> kf = kf_next;
            kf_next = load_frag<T, R>(Kb, (tile + kRadixWaves) * 32, L, lane);
            const floatx16_t acc = score_tile<T, R>(kf, qf);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const uint32_t key = score_key(acc[v]);
                if (key - base < width) park(key);
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
            if (j0 + tile_pos(v) + 4 * half < L && key - base < width) park(key);
        }
    }
    __syncthreads();

    // the r-th largest of a query's parked keys: the key x with #(y > x) < r <= #(y >= x)
    const int q = threadIdx.x / TPQ, t = threadIdx.x % TPQ;
    if (q0 + q < Lq && win[g0 + q] != 0u && ccnt[q] <= kWindowCap) {
        const int c = ccnt[q];
        const int r = krem[g0 + q];
        for (int i = t; i < c; i += TPQ) {
            const uint32_t x = cand[q][i];
            int gt = 0, eq = 0;
            for (int y = 0; y < c; ++y) {
                const uint32_t yk = cand[q][y];
                gt += yk > x;
                eq += yk == x;
            }
            if (gt < r && r <= gt + eq) {  // every thread that finds it writes the same values
                const int want = r - gt;
                prefix[g0 + q] = x;
                krem[g0 + q] = want == eq ? -want : want;
            }
        }
    }
}

// ------------------------------------------------------------------------------------ host

template <typename T, int R>
static dsv_status window_search_t(const dsv_problem &p, int Lq, const HeadTable &tab, const void *Qlr, const void *Klr,
                                  const SelectBuffers &b, hipStream_t st)
{
    const T *Ql = (const T *)Qlr;
    const T *Kl = (const T *)Klr;
    const int qtiles = (Lq + 31) / 32;
    WindowRanks wr{};
    for (int s = 0; s < tab.n; ++s) {
        const int n = window_sample_keys(p.L, tab.k[s], true);
        if (n == 0) return DSV_EINVAL;  // the caller only passes heads the search fits
        wr.tiles[s] = n / 32;
        wr.stride[s] = p.L / n;
        sample_ranks(p.L, tab.k[s], n, wr.hi[s], wr.lo[s]);
    }
    dim3 grid(qtiles, tab.n);
    hipLaunchKernelGGL((window_sample_kernel<T, R>), grid, dim3(64 * kRadixWaves), 0, st, Ql, Kl, Lq, p.L, tab, wr, b.prefix, b.win, b.todo);
    hipLaunchKernelGGL((window_hist_kernel<T, R>), grid, dim3(64 * kRadixWaves), 0, st, Ql, Kl, Lq, p.L, tab, b.prefix, b.win,
                       b.krem, b.todo, qtiles);
    hipLaunchKernelGGL((window_collect_kernel<T, R>), grid, dim3(64 * kRadixWaves), 0, st, Ql, Kl, Lq, p.L, tab, b.prefix,
                       (const uint32_t *)b.win, b.krem);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_window_search(const dsv_problem &p, int Lq, const HeadTable &tab, const void *Qlr, const void *Klr,
                                const SelectBuffers &b, hipStream_t st)
{
#define DSV_CASE(TT, RR) return window_search_t<TT, RR>(p, Lq, tab, Qlr, Klr, b, st)
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
