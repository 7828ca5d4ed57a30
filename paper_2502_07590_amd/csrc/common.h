// Shared device/host helpers of libdsv (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dsv.h"

namespace dsv {

// bf16 tensors are handled as raw 16-bit patterns.
typedef uint16_t bf16_t;

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;

constexpr int kWave = 64;
constexpr int kMaxSlots = 64;  // (batch, head) pairs described by one kernel launch

// Per-launch table of the (batch, head) pairs a grid works on, passed by value as a kernel
// argument.  Slots are ordered by descending k so that the heaviest heads are dispatched first.
struct HeadTable {
    int32_t n;
    int32_t bh[kMaxSlots];   // b * H + h
    int32_t k[kMaxSlots];    // KV kept per query in that head
    int64_t off[kMaxSlots];  // element offset of the head's [L, k] block inside idx
};

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// Round-to-nearest-even fp32 -> bf16 for finite inputs.
__device__ __forceinline__ bf16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }

template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// Sum over the 16 lanes of a DPP row; every lane of the row ends with the total.
__device__ __forceinline__ float row16_sum(float x)
{
    // row_ror:8, :4, :2, :1 (rotations inside each group of 16 lanes)
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xF, 0xF, false));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xF, 0xF, false));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xF, 0xF, false));
    x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xF, 0xF, false));
    return x;
}

// Sum over the LPR (4, 8 or 16) consecutive lanes that share one row; every lane ends with the total.
template <int LPR> __device__ __forceinline__ float row_sum(float x)
{
    static_assert(LPR == 4 || LPR == 8 || LPR == 16, "lanes per row");
    if constexpr (LPR == 16) {
        return row16_sum(x);
    } else {
        if constexpr (LPR == 8)  // row_half_mirror: lane i <-> 7 - i inside each group of 8
            x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, false));
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));  // quad_perm [1,0,3,2]
        x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));  // quad_perm [2,3,0,1]
        return x;
    }
}

__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x128, 0xF, 0xF, false)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x124, 0xF, 0xF, false)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x122, 0xF, 0xF, false)));
    x = fmaxf(x, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x121, 0xF, 0xF, false)));
    return x;
}

// ---- a lane's share of one [d]-row: CH channels, kept as raw 32-bit words --------------------
template <typename T, int CH> struct RowChunk {
    static constexpr int NW = CH * (int)sizeof(T) / 4;
    uint32_t w[NW];
};

// How the LPR lanes of a group share a row of D elements.  A lane's chunk is made of 16-byte pieces;
// its i-th piece is the lane's slot in the row's i-th strip of LPR * 16 bytes, so that one load
// instruction of the whole group covers whole strips -- whole cache lines -- instead of every other
// 16 bytes of twice as many lines (the vector memory path charges by the lines an instruction touches).
// Chunks shorter than 16 bytes are a single piece and lie side by side.
template <typename T, int D, int LPR> struct LaneLayout {
    static constexpr int CH = D / LPR;
    static constexpr int BYTES = CH * (int)sizeof(T);
    static constexpr int PE = BYTES >= 16 ? 16 / (int)sizeof(T) : CH;  // elements per piece
    static constexpr int PIECES = CH / PE;
    static constexpr int PSB = BYTES >= 16 ? LPR * 16 : 16;            // bytes from one piece to the next
    // element offset of lane s's first piece inside the row
    __device__ __forceinline__ static constexpr int off(int s) { return s * PE; }
    // true channel of the lane's c-th chunk element
    __device__ __forceinline__ static constexpr int channel(int s, int c) { return (c / PE) * (LPR * PE) + s * PE + c % PE; }
};

// The chunks of a group's lanes must tile the row: every channel owned by exactly one (lane, element).
template <typename T, int D, int LPR> constexpr bool lane_layout_tiles_the_row()
{
    typedef LaneLayout<T, D, LPR> LL;
    bool seen[D] = {};
    for (int s = 0; s < LPR; ++s)
        for (int c = 0; c < LL::CH; ++c) {
            const int ch = (c / LL::PE) * (LPR * LL::PE) + s * LL::PE + c % LL::PE;  // = LL::channel(s, c)
            if (ch < 0 || ch >= D || seen[ch]) return false;
            seen[ch] = true;
        }
    return true;
}
static_assert(lane_layout_tiles_the_row<uint16_t, 128, 4>() && lane_layout_tiles_the_row<uint16_t, 128, 8>() &&
              lane_layout_tiles_the_row<uint16_t, 128, 16>() && lane_layout_tiles_the_row<uint16_t, 64, 4>() &&
              lane_layout_tiles_the_row<uint16_t, 64, 16>() && lane_layout_tiles_the_row<float, 128, 8>() &&
              lane_layout_tiles_the_row<float, 128, 16>() && lane_layout_tiles_the_row<float, 64, 4>() &&
              lane_layout_tiles_the_row<float, 64, 8>(), "LaneLayout must be a permutation of the row's channels");

// PSB: bytes between the chunk's consecutive 16-byte pieces (16 = contiguous).
template <typename T, int CH, int PSB = 16>
__device__ __forceinline__ RowChunk<T, CH> load_chunk(const T *p)
{
    RowChunk<T, CH> c;
    constexpr int NW = RowChunk<T, CH>::NW;
    if constexpr (NW == 2) {
        uint2 v = *reinterpret_cast<const uint2 *>(p);
        c.w[0] = v.x; c.w[1] = v.y;
    } else {
        static_assert(NW % 4 == 0, "row chunk must be 8 bytes or a multiple of 16 bytes");
#pragma unroll
        for (int i = 0; i < NW / 4; ++i) {
            uint4 v = *reinterpret_cast<const uint4 *>(reinterpret_cast<const char *>(p) + i * PSB);
            c.w[4 * i + 0] = v.x; c.w[4 * i + 1] = v.y; c.w[4 * i + 2] = v.z; c.w[4 * i + 3] = v.w;
        }
    }
    return c;
}

template <typename T, int CH, int PSB = 16>
__device__ __forceinline__ void store_chunk(T *p, const float (&f)[CH])
{
    constexpr int NW = RowChunk<T, CH>::NW;
    uint32_t w[NW];
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < CH; ++i) w[i] = __float_as_uint(f[i]);
    } else {
#pragma unroll
        for (int i = 0; i < CH / 2; ++i)
            w[i] = (uint32_t)f32_to_bf16(f[2 * i]) | ((uint32_t)f32_to_bf16(f[2 * i + 1]) << 16);
    }
    if constexpr (NW == 2) {
        *reinterpret_cast<uint2 *>(p) = make_uint2(w[0], w[1]);
    } else {
#pragma unroll
        for (int i = 0; i < NW / 4; ++i)
            *reinterpret_cast<uint4 *>(reinterpret_cast<char *>(p) + i * PSB) =
                make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
    }
}

// fp32 accumulators of a lane whose chunk follows LaneLayout<T, D, LPR>, written to a plain [D] float
// row in true channel order (the partial results of the split kernels).
template <typename T, int D, int LPR>
__device__ __forceinline__ void store_acc(float *row, int s, const float (&f)[D / LPR])
{
    typedef LaneLayout<T, D, LPR> LL;
#pragma unroll
    for (int i = 0; i < LL::PIECES; ++i) {
        float *dst = row + LL::channel(s, i * LL::PE);
#pragma unroll
        for (int e = 0; e < LL::PE; e += 4)
            *reinterpret_cast<float4 *>(dst + e) = make_float4(f[i * LL::PE + e], f[i * LL::PE + e + 1], f[i * LL::PE + e + 2], f[i * LL::PE + e + 3]);
    }
}

// Partial dot product of two row chunks (this lane's CH channels), fp32 accumulation.
template <typename T, int CH>
__device__ __forceinline__ float dot_chunk(const RowChunk<T, CH> &a, const RowChunk<T, CH> &b)
{
    float acc = 0.f;
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < CH; ++i) acc = fmaf(__uint_as_float(a.w[i]), __uint_as_float(b.w[i]), acc);
    } else {
#pragma unroll
        for (int i = 0; i < CH / 2; ++i)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a.w[i]),
                                                  __builtin_bit_cast(bf16x2_t, b.w[i]), acc, false);
    }
    return acc;
}

// ---- host side ------------------------------------------------------------------------------
#define DSV_HIP_CHECK(expr)                         \
    do {                                            \
        hipError_t e_ = (expr);                     \
        if (e_ != hipSuccess) return DSV_EHIP;      \
    } while (0)

#define DSV_LAUNCH_CHECK()                                  \
    do {                                                    \
        if (hipGetLastError() != hipSuccess) return DSV_EHIP; \
    } while (0)

static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Measurement aid behind dsv_kernel_timing / dsv_kernel_ms: when switched on, a KernelSpan records one
// HIP event on the launch stream before and one after the kernel launches it encloses.
struct KernelTimer {
    bool on = false;
    hipEvent_t ev[DSV_KERNEL_COUNT][2] = {};
    bool recorded[DSV_KERNEL_COUNT] = {};
};
extern KernelTimer g_kernel_timer;
struct KernelSpan {
    int id;
    hipStream_t st;
    KernelSpan(int id_, hipStream_t st_) : id(id_), st(st_)
    {
        if (g_kernel_timer.on) (void)hipEventRecord(g_kernel_timer.ev[id][0], st);
    }
    ~KernelSpan()
    {
        if (g_kernel_timer.on) g_kernel_timer.recorded[id] = hipEventRecord(g_kernel_timer.ev[id][1], st) == hipSuccess;
    }
};

// Host: entry points of the per-stage translation units (called from api.hip).
// Lq: query rows per head in Q / Qlr (p.L for per-query selection; one proxy per group with query grouping);
// K / Klr always hold p.L rows.
dsv_status launch_project(const dsv_problem &p, int Lq, const void *Q, const void *K, const void *Wq, const void *Wk,
                          void *Qlr, void *Klr, hipStream_t st);
dsv_status launch_scores_rows(const dsv_problem &p, const void *Qlr, const void *Klr, int bh,
                              const int32_t *rows, int n_rows, float *scores, hipStream_t st);
// ---- L2-blocked (split-K) form of stage 2 -----------------------------------------------------
// Target bytes of K+V (or Q+dO) rows per key (query) range, against a 4 MB L2 per XCD.  Measured at
// L = 128k (bf16, d = 128): the forward runs best with 2 MB ranges (32 per head: 121 ms, 3 MB: 123,
// 4 MB: 124), the backward steps -- whose partial results are twice as large per range -- with 4 MB
// (dq 132 / 131 / 135 ms and dkdv 158 / 162 / 164 ms at 4 / 3 / 2 MB); 8 ranges per head are 20 % slower.
constexpr size_t kFwdRangeBytes = 2u << 20;
constexpr size_t kBwdRangeBytes = 4u << 20;
constexpr size_t kMaxRangeRows = 8192;  // rows of a range: 8 bytes of row statistics each fit 64 KB of LDS

// A key-major list of GROUPS standing for the per-query list it expands to (queries in group-major order: group g
// holds queries g G .. g G + G - 1): position pos of the expanded list is entry pos / G of the stored one, times G,
// plus pos % G.  G = 1: a plain list.  magic = floor(2^32 / G) + 1 divides positions below 2^32 / G exactly.
struct GroupExpand {
    int32_t G;
    uint32_t magic;
};
__host__ __device__ __forceinline__ GroupExpand no_expand() { return GroupExpand{1, 0u}; }
__host__ __forceinline__ GroupExpand make_expand(int G) { return GroupExpand{G, (uint32_t)((1ull << 32) / (uint64_t)G) + 1u}; }
__device__ __forceinline__ int32_t expanded_entry(const int32_t *__restrict__ list, int pos, const GroupExpand &ge)
{
    if (ge.G == 1) return list[pos];
    const int q = (int)__umulhi((uint32_t)pos, ge.magic);
    return list[q] * ge.G + (pos - q * ge.G);
}

struct SplitPlan {
    int range_len;  // keys (queries) per range
    int S;          // ranges
    int S_pad;      // S rounded up to a multiple of 8 (one XCD per residue class)
    int nqb;        // row blocks per range (each kernel sets it from its own rows per block)
};
SplitPlan make_split_plan(const dsv_problem &p, size_t range_bytes);

struct FwdSplitWorkspace {
    int32_t *seg;  // [B*H, L, S+1] segment pointers into every idx row
    float *pm;     // [B*H, L, S]    partial running max (log2 domain)
    float *pl;     // [B*H, L, S]    partial normaliser
    float *pacc;   // [B*H, L, S, d] partial unnormalised output
    int32_t *hist;   // [B*H, S, range_len + 1]  rows per segment length (then their start offsets)
    int32_t *order;  // [B*H, S, L]  rows of every (head, range) by descending segment length
};
dsv_status launch_sparse_fwd_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                   const void *K, const void *V, const int32_t *idx, void *O, float *lse,
                                   const SplitPlan &pl, const FwdSplitWorkspace &w, hipStream_t st);

// Scratch of one split backward step (dq: A, B, Delta partials; dkdv: dK, dV partials).
struct BwdSplitWorkspace {
    int32_t *seg;   // [B*H, L, S+1]
    float *pa;      // [B*H, L, S, d]
    float *pb;      // [B*H, L, S, d]
    float *pdelta;  // [B*H, L, S]   (dq step only)
    int32_t *hist;  // [B*H, S, range_len + 1]  rows per segment length (then their start offsets)
    int32_t *order; // [B*H, S, L]   rows of every (head, range) by descending segment length
    float2 *rowstat;  // [B*H, L]    {lse * log2(e), Delta} per query (dkdv step only)
};
dsv_status launch_bwd_dq_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                               const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO,
                               void *dQ, float *delta, const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st);
dsv_status launch_bwd_dkdv_split(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q,
                                 const void *K, const void *V, const int32_t *idxT, const int64_t *col,
                                 const float *lse, const float *delta, const void *dO, void *dK, void *dV,
                                 const SplitPlan &pl, const BwdSplitWorkspace &w, hipStream_t st, int expand_G = 1);
// expand_G > 1: idxT / col hold lists of groups of expand_G queries (tabs[].off the offsets of those lists); the sweep
// runs on the per-query lists they stand for.  Needs p.L < 2^32 / expand_G.

// Device buffers of the selection.  idx_t == nullptr skips the key-major emission (then jcut, cnt,
// col may be null as well).
struct SelectBuffers {
    uint32_t *prefix;  // [B*H, L]   order-preserving key of each query's threshold score
    int32_t *krem;     // [B*H, L]   number of keys equal to the threshold that belong to the top-k
    int32_t *idx;      // out: ragged query-major index
    int32_t *jcut;     // [B*H, L]   index of the last tie taken
    int32_t *tile_flag;  // [B*H, ceil(L/32)]  1: every query of the tile takes all its threshold ties
    int32_t *cnt;      // [B*H, L]   list length of every key
    int64_t *col;      // out: [B*H, L+1]
    int32_t *idx_t;    // out: ragged key-major index
    uint32_t *win;     // [B*H, L]   windowed threshold search: upper end of the bracket, then the bin width
    int32_t *todo;     // [1 + B*H * ceil(L/32)]  windowed search: number and ids of the query tiles left to the radix search
};
// Lq index rows per head (state arrays are [B*H, padded_len(Lq)], tile_flag [B*H, ceil(Lq/32)], lists hold row
// numbers below Lq); tabs[].off must be the offsets of [Lq, k] blocks.
dsv_status launch_select(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                         const SelectBuffers &b, hipStream_t st);
// Threshold search in two sweeps (stage1_window.hip) for the head slots of one table; the tiles it lists in
// b.todo still need the radix passes.
dsv_status launch_window_search(const dsv_problem &p, int Lq, const HeadTable &tab, const void *Qlr, const void *Klr,
                                const SelectBuffers &b, hipStream_t st);
// Keys the search would sample for a head keeping k of L keys, 0 if it does not fit that head (forced: leave
// out the checks that only decide whether it pays).
int window_sample_keys(int L, int k, bool forced);
// 0: automatic; 1: always the four-pass radix search; 2: the windowed search wherever it fits.  Returns the old mode
// (mode < 0: only that).
int set_threshold_search(int mode);
dsv_status launch_emit(const dsv_problem &p, int Lq, const HeadTable *tabs, int n_tabs, const void *Qlr, const void *Klr,
                       const SelectBuffers &b, hipStream_t st);
dsv_status launch_sparse_fwd(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                             const void *V, const int32_t *idx, void *O, float *lse, hipStream_t st);
dsv_status launch_bwd_dq(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                         const void *V, const int32_t *idx, const void *O, const float *lse, const void *dO, void *dQ,
                         float *delta, hipStream_t st);
dsv_status launch_bwd_dkdv(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const void *Q, const void *K,
                           const void *V, const int32_t *idxT, const int64_t *col, const float *lse, const float *delta,
                           const void *dO, void *dK, void *dV, hipStream_t st);
// ---- query grouping (grouped.hip) -----------------------------------------------------------------------
struct GroupGeom {
    int F, Hh, Ww, gf, gh, gw;
    int nh, nw;  // cubes along height and width
    int G;       // queries per group
};
// mode 0: out [B*H, L/G, d] = the groups' centre query rows; 1: out [B*H, L, d] = rows in group-major order;
// 2: the inverse of 1.
dsv_status launch_group_rows(const dsv_problem &p, const dsv_grouping &gr, int mode, const void *in, void *out,
                             hipStream_t st);
dsv_status launch_group_scalar(const dsv_problem &p, const dsv_grouping &gr, const float *in, float *out, hipStream_t st,
                               bool inverse = false);
// tabs: built for L/G rows per head.  Writes the per-query form (group-major query order) of the key-major index
// (unless idx_t_x / col_x are null) and of the query-major index (unless idx_x is null).
dsv_status launch_group_expand(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                               const int32_t *idx_g, const int32_t *idx_t_g, const int64_t *col, int32_t *idx_x,
                               int32_t *idx_t_x, int64_t *col_x, hipStream_t st);
// Group-size profiling: overlap[bh] = share of the members' own rows (per-query idx, tabs for L rows per head) that the
// centre's row holds.  count: one 64-bit counter per (b, h).
dsv_status launch_group_overlap(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                                const int32_t *idx, unsigned long long *count, float *overlap, hipStream_t st);
// Scratch of the L2-blocked grouped kernels (null seg: plain form, rows in any order).
struct GroupedSplit {
    SplitPlan plan;
    int32_t *seg;   // [B*H, L/G, S+1]
    float *pa;      // forward: pm [rows, S];          dq: C partials [rows, S, d]
    float *pb;      // forward: pl [rows, S];          dq: B partials [rows, S, d]
    float *pc;      // forward: pacc [rows, S, d];     dq: Delta partials [rows, S]
};
dsv_status launch_grouped_fwd(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                              const void *Q, const void *K, const void *V, const int32_t *idx_g, void *O, float *lse,
                              const GroupedSplit *split, hipStream_t st);
dsv_status launch_grouped_dq(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                             const void *Q, const void *K, const void *V, const int32_t *idx_g, const void *O,
                             const float *lse, const void *dO, void *dQ, float *delta, const GroupedSplit *split,
                             hipStream_t st);
dsv_status launch_row_segments(const dsv_problem &p, int rows, const HeadTable *tabs, int n_tabs, const SplitPlan &pl,
                               const int32_t *index, int32_t *seg, hipStream_t st);
dsv_status launch_fwd_merge_bf16_128(const dsv_problem &p, const float *pm, const float *pl_, const float *pacc, void *O,
                                     float *lse, int S, hipStream_t st);
dsv_status launch_dq_merge_bf16_128(const dsv_problem &p, const float *pa, const float *pb, const float *pdelta,
                                    const void *O, const void *dO, void *dQ, float *delta, int S, hipStream_t st);

// ---- predictor side (predictor.hip) ---------------------------------------------------------------------
struct PredictorLayout {
    int tok_per_block, nblk, nchunk;
    size_t part, M, T1, T2, qlr, g, ca, ch, terms, dwq, n1, n2, total;
};
PredictorLayout predictor_layout(const dsv_problem &p, int n_rows);
dsv_status launch_predictor_loss(const dsv_problem &p, const void *Q, const void *K, const void *Wq, const void *Wk,
                                 const int32_t *rows, int n, float *loss, float *dWq, float *dWk, char *ws,
                                 const PredictorLayout &w, hipStream_t st);

// ---- sparsity profiler (profiler.hip) ----------------------------------------------------------------------
size_t profile_workspace_bytes(const dsv_problem &p, int n_rows);
dsv_status launch_profile_sparsity(const dsv_problem &p, const void *Q, const void *K, const int32_t *rows, int n,
                                   float mass, int32_t *counts, float *sparsity, float *ema, float alpha, char *ws,
                                   hipStream_t st);

// report_dev: two 64-bit counters in device memory; report_host: optional HOST int64 [3].  Waits for the stream.
dsv_status launch_idx_validate(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const int32_t *idx,
                               unsigned long long *report_dev, int64_t *report_host, hipStream_t st);
// Stable transposition: every list ascending in the query index, the same result from run to run.
// cnt: scratch of idx_transpose_bytes(p) bytes (per-key totals, then per-(query chunk, key) counters); col: [B*H, L+1] int64.
size_t idx_transpose_bytes(const dsv_problem &p);
dsv_status launch_idx_transpose(const dsv_problem &p, const HeadTable *tabs, int n_tabs, const int32_t *idx,
                                int32_t *idxT, int64_t *col, int32_t *cnt, size_t cnt_bytes, hipStream_t st);

}  // namespace dsv
