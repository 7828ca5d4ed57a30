// Score tiles of stage 1 (paper Sec. "Critical KV Estimation with Kernel Fusion"): one 32x32 block of
// the low-rank product Q_lr K_lr^T per MFMA (bf16: v_mfma_f32_32x32x16_bf16, one per 16 ranks; fp32:
// v_mfma_f32_32x32x2_f32, one per 2 ranks), recomputed wherever it is needed -- never stored.
//
// Every kernel of stage 1 forms a score through score_tile() below from the same two fragments, so a
// given (query, key) pair has the same fp32 bits in every pass.  That also holds when the two
// operands trade places (rows <-> columns): the matrix cores form each output element from the same
// products in the same order either way, which the key-major emission relies on and the parity tests
// check (the transposed index must equal the transpose of the index, bit for bit).
#pragma once

#include "common.h"

namespace dsv {

// MFMA operand fragment of 32 rows of a [*, R] low-rank matrix.  Lane l holds row (l % 32) and the
// K-slice selected by (l / 32).  With fragments `rows` (A operand) and `cols` (B operand),
// acc[v] of lane l is the score of column (l % 32) against row 8*(v/4) + 4*(l/32) + (v%4).
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
__device__ __forceinline__ floatx16_t score_tile(const Frag<T, R> &rows, const Frag<T, R> &cols)
{
    floatx16_t acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = 0.f;
    if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int m = 0; m < R / 16; ++m)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(rows.v[m], cols.v[m], acc, 0, 0, 0);
    } else {
#pragma unroll
        for (int m = 0; m < R / 2; ++m)
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(rows.v[m], cols.v[m], acc, 0, 0, 0);
    }
    return acc;
}

// Row inside a 32-row tile of accumulator v for a lane in half 0 (half 1 adds 4).
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

// Waves per block of the threshold-search kernels (one block = 32 queries, the waves stride over the key
// tiles); their 32 KB histogram allows 4 blocks per CU.
#ifndef DSV_RADIX_WAVES
#define DSV_RADIX_WAVES 8
#endif
constexpr int kRadixWaves = DSV_RADIX_WAVES;

// Per-query selection state (threshold, tie budget, jcut) is stored [B*H, padded_len(L)]: rows padded
// to whole 32-query tiles, so that a tile's 32 values can be fetched with aligned vector loads.
__host__ __device__ __forceinline__ constexpr int padded_len(int L) { return (L + 31) & ~31; }

// jcut value of a query all of whose threshold-equal keys are selected: "score >= tau" decides.
constexpr int32_t kAllTies = 0x7FFFFFFF;

}  // namespace dsv
