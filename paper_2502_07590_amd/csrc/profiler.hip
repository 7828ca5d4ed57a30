// Sparsity profiler (paper Sec. "Sparsity Profiling"; definition of critical KV and head sparsity in Sec.
// "Exploiting Dynamic Sparsity"): on a sample of query rows, how many of the highest-probability keys hold
// `mass` (the paper: 90 %) of each query's softmax; the head's sparsity is the mean fraction of the other keys.
//
// Same machinery as the selection of stage 1, on the TRUE scores (contraction over all d channels, matrix
// cores) and with probability MASS in place of counts: a first sweep gives every sampled query its softmax
// normaliser (running maximum and sum); four sweeps then find, digit by digit on the order-preserving bit
// pattern of the score, the score at which the cumulative probability -- taken from the top -- reaches the
// target, histogramming count and mass per digit in LDS; the last bucket holds keys of one score, of which
// ceil(missing mass / their probability) are needed.  Scores are recomputed in every sweep, never stored.
// The mass sums come from LDS float atomics, so their last bits vary from run to run: a count can differ
// by one key when the cumulative mass passes the target within rounding of a key boundary.
#include <algorithm>

#include "stage1_core.h"

namespace dsv {

constexpr int kProfWaves = 8;

template <typename T, int D>
__device__ __forceinline__ Frag<T, D> load_query_frag(const T *__restrict__ Qh, const int32_t *__restrict__ rows, int q0,
                                                      int n, int L, int lane)
{
    const int i = min(q0 + (lane & 31), n - 1);
    return load_frag_row<T, D>(Qh, (int64_t)min(max(rows[i], 0), L - 1), lane);
}

// ---- sweep 0: softmax normaliser of every sampled query -------------------------------------------------
// stat[bh, i] = {m2, 1 / z}: m2 = max_j (s_ij * c2) (log2 domain, c2 = scale * log2 e), z = sum_j 2^(s_ij c2 - m2).
template <typename T, int D>
__global__ __launch_bounds__(64 * kProfWaves) void profile_norm_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                       const int32_t *__restrict__ rows, int n, int L,
                                                                       float c2, float2 *__restrict__ stat)
{
    __shared__ float red_m[kProfWaves][64], red_z[kProfWaves][64];
    const int bh = blockIdx.y;
    const int q0 = blockIdx.x * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int half = lane >> 5;
    const T *Qh = Q + (int64_t)bh * L * D;
    const T *Kh = K + (int64_t)bh * L * D;
    const Frag<T, D> qf = load_query_frag<T, D>(Qh, rows, q0, n, L, lane);
    const int ntiles = (L + 31) >> 5;
    float m = -INFINITY, z = 0.f;
    for (int tile = wave; tile < ntiles; tile += kProfWaves) {
        const int j0 = tile * 32;
        const Frag<T, D> kf = load_frag<T, D>(Kh, j0, L, lane);
        const floatx16_t acc = score_tile<T, D>(kf, qf);
        float s[16], mt = -INFINITY;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            s[v] = j0 + tile_pos(v) + 4 * half < L ? acc[v] * c2 : -INFINITY;
            mt = fmaxf(mt, s[v]);
        }
        const float mn = fmaxf(m, mt);
        if (mn > -INFINITY) {  // a lane whose 16 keys all lie past the end has seen nothing yet
            float add = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) add += __builtin_amdgcn_exp2f(s[v] - mn);
            z = z * __builtin_amdgcn_exp2f(m - mn) + add;   // m = -inf on the first tile: factor 0
            m = mn;
        }
    }
    red_m[wave][lane] = m;
    red_z[wave][lane] = z;
    __syncthreads();
    if (threadIdx.x < 32 && q0 + (int)threadIdx.x < n) {
        float mm = -INFINITY;
        for (int w = 0; w < kProfWaves; ++w) mm = fmaxf(mm, fmaxf(red_m[w][threadIdx.x], red_m[w][threadIdx.x + 32]));
        float zz = 0.f;
        for (int w = 0; w < kProfWaves; ++w)
            for (int h = 0; h < 2; ++h) {
                const float mw = red_m[w][threadIdx.x + 32 * h];
                if (mw > -INFINITY) zz += red_z[w][threadIdx.x + 32 * h] * __builtin_amdgcn_exp2f(mw - mm);
            }
        stat[(int64_t)bh * padded_len(n) + q0 + threadIdx.x] = make_float2(mm, 1.f / zz);
    }
}

// ---- sweeps 1-4: one digit of the threshold score ---------------------------------------------------------
// Per sampled query: prefix (digits found so far), mass_above / count_above (probability and number of keys in
// the buckets above the prefix's).  PASS 3 also writes the count of critical keys.
template <typename T, int D, int PASS>
__global__ __launch_bounds__(64 * kProfWaves) void profile_pass_kernel(const T *__restrict__ Q, const T *__restrict__ K,
                                                                       const int32_t *__restrict__ rows, int n, int L,
                                                                       float c2, float target,
                                                                       const float2 *__restrict__ stat,
                                                                       uint32_t *__restrict__ prefix,
                                                                       float *__restrict__ mass_above,
                                                                       int32_t *__restrict__ count_above,
                                                                       int32_t *__restrict__ counts)
{
    constexpr int SHIFT = 24 - 8 * PASS;
    extern __shared__ uint32_t lds[];          // [256 digits][32 queries] counts, then the same of masses
    uint32_t *hcnt = lds;
    float *hmass = reinterpret_cast<float *>(lds + 256 * 32);
    const int bh = blockIdx.y;
    const int q0 = blockIdx.x * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nq = lane & 31, half = lane >> 5;
    const T *Qh = Q + (int64_t)bh * L * D;
    const T *Kh = K + (int64_t)bh * L * D;
    for (int e = threadIdx.x; e < 2 * 256 * 32; e += 64 * kProfWaves) lds[e] = 0u;
    __syncthreads();
    const int64_t g = (int64_t)bh * padded_len(n) + min(q0 + nq, n - 1);
    const float2 st = stat[g];
    uint32_t pre = 0;
    if constexpr (PASS > 0) pre = prefix[g];
    const Frag<T, D> qf = load_query_frag<T, D>(Qh, rows, q0, n, L, lane);
    const int ntiles = (L + 31) >> 5;
    for (int tile = wave; tile < ntiles; tile += kProfWaves) {
        const int j0 = tile * 32;
        const Frag<T, D> kf = load_frag<T, D>(Kh, j0, L, lane);
        const floatx16_t acc = score_tile<T, D>(kf, qf);
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const uint32_t key = score_key(acc[v]);
            bool ok = j0 + tile_pos(v) + 4 * half < L;
            if constexpr (PASS > 0) ok = ok && ((key >> (SHIFT + 8)) == (pre >> (SHIFT + 8)));
            if (ok) {
                const uint32_t slot = ((key >> SHIFT) & 255u) * 32 + nq;
                atomicAdd(&hcnt[slot], 1u);
                atomicAdd(&hmass[slot], __builtin_amdgcn_exp2f(acc[v] * c2 - st.x) * st.y);
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < 32 && q0 + (int)threadIdx.x < n) {
        const int64_t gq = (int64_t)bh * padded_len(n) + q0 + threadIdx.x;
        float ma = PASS == 0 ? 0.f : mass_above[gq];
        int ca = PASS == 0 ? 0 : count_above[gq];
        int digit = 0;
        for (int b = 255; b >= 0; --b) {
            const float mb = hmass[b * 32 + threadIdx.x];
            const int cb = (int)hcnt[b * 32 + threadIdx.x];
            // the cumulative mass reaches the target inside this bucket (b == 0: rounding left the total a hair short)
            if ((cb > 0 && ma + mb >= target) || b == 0) { digit = b; break; }
            ma += mb;
            ca += cb;
        }
        const uint32_t full = (PASS == 0 ? 0u : prefix[gq]) | ((uint32_t)digit << SHIFT);
        prefix[gq] = full;
        mass_above[gq] = ma;
        count_above[gq] = ca;
        if constexpr (PASS == 3) {
            // every key of this bucket has the score `full` decodes to, hence the same probability
            const int cb = max((int)hcnt[digit * 32 + threadIdx.x], 1);
            const float2 s2 = stat[gq];
            const float p = __builtin_amdgcn_exp2f(key_score(full) * c2 - s2.x) * s2.y;
            int need = p > 0.f ? (int)ceilf((target - ma) / p) : cb;
            need = min(max(need, 1), cb);
            counts[(int64_t)bh * n + q0 + threadIdx.x] = ca + need;
        }
    }
}

// sparsity[bh] = mean_i (1 - counts_i / L); ema[bh] = alpha * sparsity + (1 - alpha) * ema[bh] when ema is given.
__global__ __launch_bounds__(256) void profile_finish_kernel(const int32_t *__restrict__ counts, int n, int L,
                                                             float *__restrict__ sparsity, float *__restrict__ ema,
                                                             float alpha)
{
    __shared__ double part[256];
    const int bh = blockIdx.x;
    double s = 0.0;
    for (int i = threadIdx.x; i < n; i += 256) s += 1.0 - (double)counts[(int64_t)bh * n + i] / (double)L;
    part[threadIdx.x] = s;
    __syncthreads();
    for (int step = 128; step; step >>= 1) {
        if ((int)threadIdx.x < step) part[threadIdx.x] += part[threadIdx.x + step];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const float p = (float)(part[0] / (double)n);
        sparsity[bh] = p;
        if (ema) ema[bh] = alpha * p + (1.f - alpha) * ema[bh];
    }
}

// ------------------------------------------------------------------------------------ host
template <typename T, int D>
static dsv_status profile_t(const dsv_problem &p, const void *Q, const void *K, const int32_t *rows, int n, float mass,
                            int32_t *counts, float *sparsity, float *ema, float alpha, char *ws, hipStream_t st)
{
    const int nbh = p.B * p.H;
    const size_t np_ = (size_t)nbh * padded_len(n);
    float2 *stat = reinterpret_cast<float2 *>(ws);
    uint32_t *prefix = reinterpret_cast<uint32_t *>(ws + align_up(np_ * 8, 256));
    float *mabove = reinterpret_cast<float *>(reinterpret_cast<char *>(prefix) + align_up(np_ * 4, 256));
    int32_t *cabove = reinterpret_cast<int32_t *>(reinterpret_cast<char *>(mabove) + align_up(np_ * 4, 256));
    const float c2 = p.scale * 1.4426950408889634f;
    const size_t lds = 2 * 256 * 32 * 4;
    static bool attr_set = false;  // the histogram pair needs 64 KB of dynamic LDS
    if (!attr_set) {
        DSV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&profile_pass_kernel<T, D, 0>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        DSV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&profile_pass_kernel<T, D, 1>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        DSV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&profile_pass_kernel<T, D, 2>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        DSV_HIP_CHECK(hipFuncSetAttribute(reinterpret_cast<const void *>(&profile_pass_kernel<T, D, 3>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    dim3 grid((n + 31) / 32, nbh), block(64 * kProfWaves);
    hipLaunchKernelGGL((profile_norm_kernel<T, D>), grid, block, 0, st, (const T *)Q, (const T *)K, rows, n, p.L, c2, stat);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL((profile_pass_kernel<T, D, 0>), grid, block, lds, st, (const T *)Q, (const T *)K, rows, n, p.L, c2, mass, stat, prefix, mabove, cabove, counts);
    hipLaunchKernelGGL((profile_pass_kernel<T, D, 1>), grid, block, lds, st, (const T *)Q, (const T *)K, rows, n, p.L, c2, mass, stat, prefix, mabove, cabove, counts);
    hipLaunchKernelGGL((profile_pass_kernel<T, D, 2>), grid, block, lds, st, (const T *)Q, (const T *)K, rows, n, p.L, c2, mass, stat, prefix, mabove, cabove, counts);
    hipLaunchKernelGGL((profile_pass_kernel<T, D, 3>), grid, block, lds, st, (const T *)Q, (const T *)K, rows, n, p.L, c2, mass, stat, prefix, mabove, cabove, counts);
    DSV_LAUNCH_CHECK();
    hipLaunchKernelGGL(profile_finish_kernel, dim3(nbh), dim3(256), 0, st, counts, n, p.L, sparsity, ema, alpha);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

size_t profile_workspace_bytes(const dsv_problem &p, int n)
{
    const size_t np_ = (size_t)p.B * p.H * padded_len(n);
    return align_up(np_ * 8, 256) + 3 * align_up(np_ * 4, 256);
}

dsv_status launch_profile_sparsity(const dsv_problem &p, const void *Q, const void *K, const int32_t *rows, int n,
                                   float mass, int32_t *counts, float *sparsity, float *ema, float alpha, char *ws,
                                   hipStream_t st)
{
    if (p.dtype == DSV_BF16) {
        if (p.d == 64) return profile_t<bf16_t, 64>(p, Q, K, rows, n, mass, counts, sparsity, ema, alpha, ws, st);
        if (p.d == 128) return profile_t<bf16_t, 128>(p, Q, K, rows, n, mass, counts, sparsity, ema, alpha, ws, st);
    } else if (p.dtype == DSV_F32) {
        if (p.d == 64) return profile_t<float, 64>(p, Q, K, rows, n, mass, counts, sparsity, ema, alpha, ws, st);
        if (p.d == 128) return profile_t<float, 128>(p, Q, K, rows, n, mass, counts, sparsity, ema, alpha, ws, st);
    }
    return DSV_EUNSUPPORTED;
}

}  // namespace dsv
