// Query grouping (paper Sec. "Sparse Attention with Query Grouping"; Observation 5): the queries of a
// 3D cube of the frames x height x width token grid share ONE index row, chosen by the cube's centre
// query.  Stage 1 then scores only one query per group; stage 2 gathers every selected K / V row once per
// group and uses it for all G members, which turns the per-query gather sweep (one K row and one V row
// per (query, key) pair, ~1 flop per byte) into small dense tiles.
//
// Forward kernel (bf16, d = 128): one wave per 8 queries of a group (groups of up to 32 queries: up to four waves that
// share the gathered rows).
//   scores   S[q, key] for 32 keys at a time on the matrix cores: A = the group's query rows (rows >= G are
//            zero), B = the 32 gathered K rows, one v_mfma_f32_32x32x16_bf16 per 16 channels.  Lane l then
//            holds key (l % 32) against queries 4 * (l / 32) + 0..3 (accumulators 0..3; the other twelve
//            belong to the zero rows and are ignored).
//   softmax  online, in the log2 domain; the tile maximum of a query is a reduction over the 32 lanes of a
//            half-wave.  Probabilities go to LDS as bf16 [query][key slot].
//   output   O[q, :] += p[q, key] * V[key, :] on the matrix cores as well (v_mfma_f32_16x16x32_bf16, the
//            contraction over the tile's 32 keys), the gathered V rows transposed on their way through LDS.
// Bytes through the vector memory path per (query, key) pair: (256 + 256) / G + 4 / G instead of 516.
#include <algorithm>

#include "stage2_core.h"

namespace dsv {

// Member m of group g -> token index (frames first, then height, then width; groups and members in the
// same order).
__device__ __forceinline__ int64_t member_token(const GroupGeom &gm, int g, int m)
{
    const int cw = g % gm.nw, ch = (g / gm.nw) % gm.nh, cf = g / (gm.nw * gm.nh);
    const int mw = m % gm.gw, mh = (m / gm.gw) % gm.gh, mf = m / (gm.gw * gm.gh);
    return ((int64_t)(cf * gm.gf + mf) * gm.Hh + (ch * gm.gh + mh)) * gm.Ww + (cw * gm.gw + mw);
}

typedef uint16_t __attribute__((may_alias)) u16_alias;
typedef uint32_t __attribute__((may_alias)) u32_alias;
typedef float __attribute__((may_alias)) f32_alias;

// LDS traffic between the lanes of ONE wave: keeps the compiler from moving accesses across the point.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ float half_max(float x)  // over the 32 lanes of a half-wave
{
    x = row16_max(x);
    return fmaxf(x, __shfl_xor(x, 16));
}
__device__ __forceinline__ float half_sum(float x)
{
    x = row16_sum(x);
    return x + __shfl_xor(x, 16);
}

// ---- rows of [B*H, L, D] gathered into [B*H, n_out, D]: out[bh, r] = in[bh, src(r)] --------------------
//   MODE 0: r = group,            src = the group's centre query          (n_out = L / G)
//   MODE 1: r = g * G + m,        src = member m of group g               (n_out = L): group-major order
//   MODE 2: the inverse of MODE 1: out[bh, member(g, m)] = in[bh, g * G + m]
template <typename T, int MODE>
__global__ __launch_bounds__(256) void group_rows_kernel(const T *__restrict__ in, T *__restrict__ out, int L, int D,
                                                         int n_out, GroupGeom gm, int centre)
{
    const int per_row = D * (int)sizeof(T) / 16;  // 16-byte pieces per row
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int bh = blockIdx.y;
    if (e >= (int64_t)n_out * per_row) return;
    const int r = (int)(e / per_row), piece = (int)(e % per_row);
    int64_t src, dst;
    if (MODE == 0) { src = member_token(gm, r, centre); dst = r; }
    else if (MODE == 1) { src = member_token(gm, r / gm.G, r % gm.G); dst = r; }
    else { src = r; dst = member_token(gm, r / gm.G, r % gm.G); }
    const int n_in = MODE == 0 ? L : n_out;
    const uint4 *s = reinterpret_cast<const uint4 *>(in + ((int64_t)bh * n_in + src) * D) + piece;
    uint4 *d = reinterpret_cast<uint4 *>(out + ((int64_t)bh * n_out + dst) * D) + piece;
    *d = *s;
}

// lse (one float per token) into group-major order, or (inverse) back into token order.
__global__ __launch_bounds__(256) void group_scalar_kernel(const float *__restrict__ in, float *__restrict__ out, int L,
                                                           GroupGeom gm, int inverse)
{
    const int r = blockIdx.x * 256 + threadIdx.x;
    const int bh = blockIdx.y;
    if (r >= L) return;
    const int64_t tok = member_token(gm, r / gm.G, r % gm.G);
    if (inverse) out[(int64_t)bh * L + tok] = in[(int64_t)bh * L + r];
    else out[(int64_t)bh * L + r] = in[(int64_t)bh * L + tok];
}

// ---- the per-query index the grouped one stands for, in group-major query order ------------------------
// idx_x[bh][g * G + m][:] = idx_g[bh][g][:]
__global__ __launch_bounds__(256) void expand_idx_kernel(const int32_t *__restrict__ idx_g, int32_t *__restrict__ idx_x,
                                                         int Lq, int G, HeadTable tab)
{
    const int slot = blockIdx.y;
    const int k = tab.k[slot];
    const int32_t *src = idx_g + tab.off[slot];           // [Lq, k]
    int32_t *dst = idx_x + tab.off[slot] * G;              // [Lq * G, k]
    for (int64_t g = blockIdx.x; g < Lq; g += gridDim.x)
        for (int t = threadIdx.x; t < k; t += 256) {
            const int32_t v = src[g * k + t];
#pragma unroll 1
            for (int m = 0; m < G; ++m) dst[(g * G + m) * k + t] = v;
        }
}

// Key-major: entry e of a list (a group g) becomes the G entries g * G + 0 .. G - 1 at positions e * G ...;
// lists of ascending groups stay ascending.  col_x = G * col.
__global__ __launch_bounds__(256) void expand_idx_t_kernel(const int32_t *__restrict__ idx_t_g,
                                                           int32_t *__restrict__ idx_t_x, int Lq, int G, HeadTable tab)
{
    const int slot = blockIdx.y;
    const int64_t n = (int64_t)Lq * tab.k[slot];
    const int32_t *src = idx_t_g + tab.off[slot];
    int32_t *dst = idx_t_x + tab.off[slot] * G;
    const int64_t stride = (int64_t)gridDim.x * 256;
    // one thread per source entry; its G outputs are contiguous (G a multiple of 4: 16-byte stores; tab.off is a multiple
    // of the row length, the output stays 16-byte aligned whenever that is a multiple of 4 entries)
    const bool wide = (G & 3) == 0 && ((tab.off[slot] * G) & 3) == 0;
    for (int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x; e < n; e += stride) {
        const int32_t b = src[e] * G;
        if (wide) {
            int4 *o = reinterpret_cast<int4 *>(dst + e * G);
            for (int m = 0; m < G; m += 4) o[m >> 2] = make_int4(b + m, b + m + 1, b + m + 2, b + m + 3);
        } else {
#pragma unroll 1
            for (int m = 0; m < G; ++m) dst[e * G + m] = b + m;
        }
    }
}

__global__ __launch_bounds__(256) void scale_col_kernel(const int64_t *__restrict__ col, int64_t *__restrict__ col_x,
                                                        int64_t n, int G)
{
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e < n) col_x[e] = col[e] * G;
}

// ---- share of the members' own selections that the centre's row holds (group-size profiling) -------------------
// One block walks groups blockIdx.x, blockIdx.x + gridDim.x, ... of one head: the centre query's row goes into a
// bitmap of L bits in LDS, every member's row is tested against it, and the row's own words are cleared again.
// count[bh] += number of (member, key) pairs found; integer sums, so the result does not depend on the order.
__global__ __launch_bounds__(256) void group_overlap_kernel(const int32_t *__restrict__ idx, int L, HeadTable tab,
                                                            GroupGeom gm, int centre,
                                                            unsigned long long *__restrict__ count)
{
    extern __shared__ uint32_t bitmap[];  // [(L + 31) / 32]
    __shared__ unsigned long long part[4];
    const int slot = blockIdx.y;
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int32_t *base = idx + tab.off[slot];
    const int Lq = L / gm.G;
    for (int w = threadIdx.x; w < (L + 31) / 32; w += 256) bitmap[w] = 0u;
    __syncthreads();
    unsigned long long mine = 0;
    for (int g = blockIdx.x; g < Lq; g += gridDim.x) {
        const int32_t *crow = base + member_token(gm, g, centre) * k;
        for (int t = threadIdx.x; t < k; t += 256) {
            const int v = crow[t];
            if (v >= 0 && v < L) atomicOr(&bitmap[v >> 5], 1u << (v & 31));
        }
        __syncthreads();
        for (int m = 0; m < gm.G; ++m) {
            const int32_t *row = base + member_token(gm, g, m) * k;
            for (int t = threadIdx.x; t < k; t += 256) {
                const int v = row[t];
                if (v >= 0 && v < L) mine += (bitmap[v >> 5] >> (v & 31)) & 1u;
            }
        }
        __syncthreads();
        for (int t = threadIdx.x; t < k; t += 256) {
            const int v = crow[t];
            if (v >= 0 && v < L) bitmap[v >> 5] = 0u;
        }
        __syncthreads();
    }
    for (int o = 32; o; o >>= 1) mine += __shfl_xor(mine, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = mine;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(&count[bh], part[0] + part[1] + part[2] + part[3]);
}

__global__ void group_overlap_reset_kernel(unsigned long long *count, int n)
{
    const int e = blockIdx.x * 256 + threadIdx.x;
    if (e < n) count[e] = 0ull;
}

__global__ void group_overlap_finish_kernel(const unsigned long long *__restrict__ count, float *__restrict__ overlap,
                                            int L, HeadTable tab)
{
    const int slot = threadIdx.x;
    if (slot < tab.n) overlap[tab.bh[slot]] = (float)((double)count[tab.bh[slot]] / ((double)L * tab.k[slot]));
}

// Linear block id -> (head slot, key range, block of 4 groups), consecutive ids on consecutive XCDs, every XCD
// walking its own ranges one after the other (the order of the per-query L2-blocked sweeps).
__device__ __forceinline__ bool decode_group_item(const SplitPlan &pl, int64_t b, int &slot, int &range, int &gb)
{
    const int64_t per_head = (int64_t)pl.S_pad * pl.nqb;
    slot = (int)(b / per_head);
    const int64_t rem = b - (int64_t)slot * per_head;
    const int xcd = (int)(rem & 7);
    const int64_t local = rem >> 3;
    const int t = (int)(local / pl.nqb);
    gb = (int)(local - (int64_t)t * pl.nqb);
    range = t * 8 + xcd;
    return range < pl.S;
}

// ---- grouped forward ------------------------------------------------------------------------------------
// Both products of a tile run on the matrix cores.
//   S = Q_g K^T   v_mfma_f32_32x32x16_bf16 per 16 channels: A = the group's query rows (rows >= G zero), B = the 32
//                 gathered K rows (lane = key, 8 channels), read from the rows parked in LDS.
//   O += P V      v_mfma_f32_16x16x32_bf16 per 16 channels: A = P (rows = queries, rows >= 8 zero), B = V with the
//                 contraction over the tile's 32 keys.  A B fragment holds, per lane, 8 KEYS of one channel -- the
//                 transpose of how a gathered row arrives -- so the tile's V rows are parked row-major in LDS and
//                 read back with transposing LDS reads (tr_frag below).  Which keys a lane group contracts is
//                 free as long as A and B agree (fwd_key below); P is stored with each group's keys contiguous,
//                 so its fragment is one 16-byte read.
// SPLIT: the L2-blocked form for ascending rows -- a block works on ONE key range (whose K + V rows stay in its
// XCD's L2), walks only the segment of every group's row that falls into the range, and leaves the partial softmax
// state (m, l, unnormalised acc) of every member for the per-query merge kernel; pm, pl_, pacc are laid out per
// TOKEN row like the per-query partials.
constexpr int kVRow = 128 * 2 + 16;  // bytes from one parked row to the next

// Transposing LDS read (ds_read_b64_tr_b16): inside every block of 16 lanes, lane i receives four halfwords, the
// e-th being halfword (i % 4) at the address passed by lane 4 e + i / 4 of the block.  So when lane 4 e + q
// passes the address of channels c0 + 4 q .. + 3 of parked row key(e), lane i ends up with channel c0 + i of rows
// key(0..3): a quarter of a matrix-core B fragment whose contraction runs over the parked rows.  Two reads
// (rows key(0..3), key(4..7)) make the 8-element fragment.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
__device__ __forceinline__ bf16x8_t tr_frag(const unsigned char *a0, const unsigned char *a1)
{
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)a0);
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)a1);
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t f = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8_t, f);
}

// Forward, O += P V: lane group g (16 lanes) contracts, in this order, keys fwd_key(g, 0..7); the 32 lanes that
// one pass of a read serves (two lane groups) then touch 8 rows 2 apart, i.e. 8 disjoint stretches of LDS banks
// (272-byte rows).  p_slot: place of key n in a row of P, where the 8 keys of a lane group are contiguous.
__device__ __forceinline__ int fwd_key(int g, int e) { return 16 * (e >> 2) + 2 * (4 * (g & 1) + (e & 3)) + (g >> 1); }
__device__ __forceinline__ int p_slot(int n) { return 16 * (n & 1) + 8 * ((n >> 3) & 1) + 4 * (n >> 4) + ((n >> 1) & 3); }

// NSUB = 1: the four waves of a block take four groups of at most 8 queries.  NSUB = 2 / 4: ONE group of up to 16 / 32
// queries per block of NSUB waves, wave w taking members 8 w .. 8 w + 7; the waves gather the tile's rows together (two load instructions
// each instead of eight), park them once, and every wave forms its own 8 members' scores and outputs from the shared
// rows -- each K / V row crosses the vector memory path once per 32 queries.
template <int D, bool SPLIT, int NSUB>
__global__ __launch_bounds__(256) void grouped_fwd_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                          const bf16_t *__restrict__ V,
                                                          const int32_t *__restrict__ idx_g, bf16_t *__restrict__ O,
                                                          float *__restrict__ lse, const int32_t *__restrict__ seg,
                                                          float *__restrict__ pm, float *__restrict__ pl_,
                                                          float *__restrict__ pacc, int L, int Lq, float scale,
                                                          HeadTable tab, GroupGeom gm, SplitPlan pl)
{
    static_assert(D == 128, "8 channel blocks of 16");
    constexpr int NM = D / 16;
    int slot, range = 0, gb;
    if (SPLIT) {
        if (!decode_group_item(pl, blockIdx.x, slot, range, gb)) return;
    } else {
        slot = blockIdx.y;
        gb = blockIdx.x;
    }
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int g = NSUB == 1 ? gb * 4 + wave : gb;
    if (g >= Lq) return;  // NSUB = 1: the whole wave leaves, nothing below synchronises across waves; else the whole block
    const int G = gm.G;
    const int mb = NSUB == 1 ? 0 : 8 * wave;     // first member this wave works for
    const bool active = mb < G;                  // NSUB = 4: waves beyond the group still load and synchronise
    const int Gw = min(G - mb, 8);               // members of this wave (<= 0: none)
    auto block_sync = [&]() { if constexpr (NSUB == 1) wave_sync(); else __syncthreads(); };
    const bf16_t *Qh = Q + (int64_t)bh * L * D;
    const bf16_t *Kh = K + (int64_t)bh * L * D;
    const bf16_t *Vh = V + (int64_t)bh * L * D;
    const int32_t *row = idx_g + tab.off[slot] + (int64_t)g * k;
    int tb = 0, te = k;
    if (SPLIT) {
        const int32_t *sp = seg + ((int64_t)bh * Lq + g) * (pl.S + 1) + range;
        tb = sp[0];
        te = sp[1];
    }

    __shared__ __align__(16) unsigned char k_all[NSUB == 1 ? 4 : 1][32 * kVRow];   // per wave, or one for the block
    __shared__ __align__(16) unsigned char v_all[NSUB == 1 ? 4 : 1][32 * kVRow];
    __shared__ __align__(16) uint32_t p_all[4][16 * 16 + 8];
    unsigned char *K_s = k_all[NSUB == 1 ? wave : 0];                        // the tile's 32 K rows, row-major
    unsigned char *V_s = v_all[NSUB == 1 ? wave : 0];                        // the tile's 32 V rows
    u32_alias *P_s = p_all[wave];                                            // [16 rows][32 key slots] bf16, rows 8.. zero
    f32_alias *fac_s = reinterpret_cast<f32_alias *>(p_all[wave] + 16 * 16);  // [8 queries]
    for (int e = lane; e < 16 * 16; e += 64) P_s[e] = 0u;

    // A operand of the scores: query row (lane % 32) of the group, zero beyond the group
    bf16x8_t qa[NM];
    {
        const int64_t tq = member_token(gm, g, min(mb + n, G - 1));
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            uint4 raw = *reinterpret_cast<const uint4 *>(Qh + tq * D + m * 16 + half * 8);
            if (n >= Gw) raw = make_uint4(0u, 0u, 0u, 0u);
            qa[m] = __builtin_bit_cast(bf16x8_t, raw);
        }
    }
    float M[4], lsum[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) { M[v] = -INFINITY; lsum[v] = 0.f; }
    floatx4_t oacc[NM];  // oacc[nb][v]: query 4 * g4 + v (lane groups 0 and 1), channel 16 nb + c16
#pragma unroll
    for (int nb = 0; nb < NM; ++nb) oacc[nb] = floatx4_t{0.f, 0.f, 0.f, 0.f};
    const float c2 = scale * kLog2e;
    const int pslot = p_slot(n);
    // this lane's addresses for the transposing reads of V: rows fwd_key(g4, c16 / 4) and fwd_key(g4, 4 + c16 / 4),
    // channels 4 (c16 % 4) .. + 3 of a 16-channel block
    const int vt0 = fwd_key(g4, c16 >> 2) * kVRow + (c16 & 3) * 8;
    const int vt1 = fwd_key(g4, 4 + (c16 >> 2)) * kVRow + (c16 & 3) * 8;

    // Gathered rows come in whole: one load instruction fetches 4 rows, 16 lanes x 16 bytes each (every 64-byte
    // sector the vector memory path moves is used in full; loading matrix-core fragments straight from memory
    // would touch 32 rows x 32 bytes per instruction and waste half of every sector).  Rows go to LDS row-major;
    // the score fragments (lane = key, 8 channels) and the transposed V fragments are read from there.
    // Software pipeline: while tile t is worked on, the rows of tile t+1 are in flight and the index entries of
    // tile t+2 are requested.  Keys past the end of the segment repeat its last entry and get probability zero.
    constexpr int NI = 8 / NSUB;                 // load instructions (4 rows each) of this wave per tile and matrix
    const int i0 = NSUB == 1 ? 0 : NI * wave;    // the first of them
    int32_t jr[NI];
    bf16x8_t kr[NI], vr[NI];
    auto load_idx = [&](int t0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) jr[i] = row[min(t0 + g4 + 4 * (i0 + i), te - 1)];
    };
    auto load_rows = [&]() {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            kr[i] = *reinterpret_cast<const bf16x8_t *>(Kh + (int64_t)jr[i] * D + c16 * 8);
            vr[i] = *reinterpret_cast<const bf16x8_t *>(Vh + (int64_t)jr[i] * D + c16 * 8);
        }
    };
    if (tb < te) {
        load_idx(tb);
        load_rows();
        if (tb + 32 < te) load_idx(tb + 32);
    }
    wave_sync();
    for (int t0 = tb; t0 < te; t0 += 32) {
        const int nvalid = min(32, te - t0);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            *reinterpret_cast<bf16x8_t *>(K_s + (g4 + 4 * (i0 + i)) * kVRow + c16 * 16) = kr[i];
            *reinterpret_cast<bf16x8_t *>(V_s + (g4 + 4 * (i0 + i)) * kVRow + c16 * 16) = vr[i];
        }
        block_sync();
        if (t0 + 32 < te) {  // wave-uniform
            load_rows();
            if (t0 + 64 < te) load_idx(t0 + 64);
        }
        floatx16_t acc;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = 0.f;
#pragma unroll
        for (int m = 0; m < NM; ++m) {
            const bf16x8_t kb = *reinterpret_cast<const bf16x8_t *>(K_s + n * kVRow + (m * 16 + half * 8) * 2);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa[m], kb, acc, 0, 0, 0);
        }
        float p[4], corr[4];
        bool moved = false;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float s = n < nvalid ? acc[v] * c2 : -INFINITY;
            const float mn = fmaxf(M[v], half_max(s));
            corr[v] = fast_exp2(M[v] - mn);
            moved = moved || (mn != M[v]);
            M[v] = mn;
            p[v] = fast_exp2(s - mn);
            lsum[v] = fmaf(lsum[v], corr[v], p[v]);
        }
        moved = __any(moved);
#pragma unroll
        for (int v = 0; v < 4; ++v) reinterpret_cast<u16_alias *>(P_s)[(4 * half + v) * 32 + pslot] = f32_to_bf16(p[v]);
        if (moved && n == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) fac_s[4 * half + v] = corr[v];
        }
        wave_sync();
        if (moved) {  // wave-uniform
            const float4 f = *reinterpret_cast<const float4 *>(const_cast<const float *>(fac_s) + 4 * (g4 & 1));
#pragma unroll
            for (int nb = 0; nb < NM; ++nb) {
                oacc[nb][0] *= f.x; oacc[nb][1] *= f.y; oacc[nb][2] *= f.z; oacc[nb][3] *= f.w;
            }
        }
        const bf16x8_t pa = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(const_cast<const uint32_t *>(P_s) + c16 * 16 + g4 * 4));
#pragma unroll
        for (int nb = 0; nb < NM; ++nb)
            oacc[nb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pa, tr_frag(V_s + vt0 + nb * 32, V_s + vt1 + nb * 32), oacc[nb], 0, 0, 0);
        block_sync();  // the next tile overwrites P_s and the parked rows
    }
    if (!active) return;
    // query 4 * half + v lives in this half-wave's softmax state; the output rows of queries 4 * g4 + v in lane groups 0, 1
    float lt[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) lt[v] = half_sum(lsum[v]);
    if (SPLIT) {
        // partial state of this (member, range); an empty segment leaves (m = -inf, l = 0, acc = 0)
        if (n == 0) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int q = 4 * half + v;
                if (q < Gw) {
                    const int64_t slot_id = ((int64_t)bh * L + member_token(gm, g, mb + q)) * pl.S + range;
                    pm[slot_id] = M[v];
                    pl_[slot_id] = lt[v];
                }
            }
        }
        if (g4 < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int q = 4 * g4 + v;
                if (q < Gw) {
                    const int64_t slot_id = ((int64_t)bh * L + member_token(gm, g, mb + q)) * pl.S + range;
#pragma unroll
                    for (int nb = 0; nb < NM; ++nb) pacc[slot_id * D + nb * 16 + c16] = oacc[nb][v];
                }
            }
        }
        return;
    }
    if (n == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int q = 4 * half + v;
            fac_s[q] = 1.f / lt[v];
            if (q < Gw) lse[(int64_t)bh * L + member_token(gm, g, mb + q)] = (M[v] + log2f(lt[v])) * kLn2;
        }
    }
    wave_sync();
    if (g4 < 2) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int q = 4 * g4 + v;
            if (q < Gw) {
                const float inv = fac_s[q];
                bf16_t *orow = O + ((int64_t)bh * L + member_token(gm, g, mb + q)) * D;
#pragma unroll
                for (int nb = 0; nb < NM; ++nb) orow[nb * 16 + c16] = f32_to_bf16(oacc[nb][v] * inv);
            }
        }
    }
}

// ---- grouped backward, dQ step -------------------------------------------------------------------------------
// Same tiling and the same row parking as the forward.  Per tile of 32 keys:
//   S = Q_g K^T and dP = dO_g V^T   v_mfma_f32_16x16x32_bf16 (16 keys x 16 query rows, 32 channels per instruction;
//        the A fragments of 8 real query rows cost 16 registers instead of the 32 of the 32-row form), B fragments
//        read from the parked rows.  Lane l < 32 then holds queries 4 (l / 16) + 0..3 against keys (l % 16) and
//        16 + (l % 16); the upper half-wave holds the zero rows.
//   per pair  p = 2^(s c2 - lse2), and the three sums of the per-query dq sweep (stage2_core.h):
//        C = sum p (dP - D0) k, B = sum p k, Delta = sum p dP, with D0 = dO . O_stored as the centring value;
//        dQ = scale (C - (Delta - D0) B).
//   C and B   one product on the matrix cores, v_mfma_f32_32x32x16_bf16 with the contraction over the keys: the 32
//        A rows are the weights p (dP - D0) of the 8 members as bf16 head and tail (rows 0..7, 8..15) and p as head
//        and tail (rows 16..23, 24..31) -- two bf16 terms carry 16 significant bits of every fp32 weight -- and B is
//        K transposed, read from the parked rows with transposing LDS reads (tr_frag; which keys a lane group
//        takes: dq_key below).
// SPLIT: per (member, range) partials C, B, Delta for the per-query dq merge kernel.

// dQ step, second product: lane group h (32 lanes) of k-step s contracts, in this order, keys dq_key(s, h, 0..7);
// one pass of a transposing read then touches 4 rows 4 apart, 64 bytes each: disjoint LDS banks.  w_slot: place
// of key n in a row of the weight matrix, where the 8 keys of (k-step, lane group) are contiguous.
__device__ __forceinline__ int dq_key(int s, int h, int e) { return 16 * s + 4 * (e & 3) + 2 * h + (e >> 2); }
__device__ __forceinline__ int w_slot(int n) { return (n & 16) + 8 * ((n >> 1) & 1) + 4 * (n & 1) + ((n >> 2) & 3); }

// x = head + tail as two bf16 values (head = x rounded to bf16, tail = the rounded remainder)
__device__ __forceinline__ void split_bf16(float x, uint16_t &hi, uint16_t &lo)
{
    hi = f32_to_bf16(x);
    lo = f32_to_bf16(x - __uint_as_float((uint32_t)hi << 16));
}

// NSUB as in the forward: 4 = one group of up to 32 queries per block, the rows gathered and parked once per block.
template <int D, bool SPLIT, int NSUB>
__global__ __launch_bounds__(256) void grouped_dq_kernel(const bf16_t *__restrict__ Q, const bf16_t *__restrict__ K,
                                                         const bf16_t *__restrict__ V, const int32_t *__restrict__ idx_g,
                                                         const bf16_t *__restrict__ O, const float *__restrict__ lse,
                                                         const bf16_t *__restrict__ dO, bf16_t *__restrict__ dQ,
                                                         float *__restrict__ delta_out, const int32_t *__restrict__ seg,
                                                         float *__restrict__ pa, float *__restrict__ pb,
                                                         float *__restrict__ pdelta, int L, int Lq, float scale,
                                                         HeadTable tab, GroupGeom gm, SplitPlan pl)
{
    static_assert(D == 128, "4 channel blocks of 32");
    constexpr int NC = D / 32;
    int slot, range = 0, gb;
    if (SPLIT) {
        if (!decode_group_item(pl, blockIdx.x, slot, range, gb)) return;
    } else {
        slot = blockIdx.y;
        gb = blockIdx.x;
    }
    const int bh = tab.bh[slot];
    const int k = tab.k[slot];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n = lane & 31, half = lane >> 5;
    const int c16 = lane & 15, g4 = lane >> 4;
    const int g = NSUB == 1 ? gb * 4 + wave : gb;
    if (g >= Lq) return;  // NSUB = 1: whole wave; else whole block
    const int G = gm.G;
    const int mb = NSUB == 1 ? 0 : 8 * wave;     // first member this wave works for
    const bool active = mb < G;
    const int Gw = min(G - mb, 8);               // members of this wave (<= 0: none; the wave still loads and synchronises)
    auto block_sync = [&]() { if constexpr (NSUB == 1) wave_sync(); else __syncthreads(); };
    const int64_t hb = (int64_t)bh * L * D;
    const bf16_t *Kh = K + hb, *Vh = V + hb;
    const int32_t *row = idx_g + tab.off[slot] + (int64_t)g * k;
    int tb = 0, te = k;
    if (SPLIT) {
        const int32_t *sp = seg + ((int64_t)bh * Lq + g) * (pl.S + 1) + range;
        tb = sp[0];
        te = sp[1];
    }
    __shared__ __align__(16) unsigned char k_all[NSUB == 1 ? 4 : 1][32 * kVRow];   // per wave, or one for the block
    __shared__ __align__(16) unsigned char v_all[NSUB == 1 ? 4 : 1][32 * kVRow];
    __shared__ __align__(16) uint32_t w_all[4][32 * 16 + 16];
    unsigned char *K_s = k_all[NSUB == 1 ? wave : 0];   // the tile's 32 K rows, row-major
    unsigned char *V_s = v_all[NSUB == 1 ? wave : 0];   // the tile's 32 V rows
    u32_alias *W_s = w_all[wave];       // [32 rows][32 key slots] bf16: weights of the second product
    f32_alias *q_s = reinterpret_cast<f32_alias *>(w_all[wave] + 32 * 16);  // [8] D0, then [8] Delta - D0

    // A operands of the score-shaped products: the members' Q and dO rows (zero beyond the group), 16-row form:
    // lane = (row l % 16, channels 32 m + 8 (l / 16) .. + 8)
    bf16x8_t qa[4], ga[4];
    {
        const int64_t tq = member_token(gm, g, min(mb + c16, G - 1));
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            uint4 rq = *reinterpret_cast<const uint4 *>(Q + hb + tq * D + m * 32 + g4 * 8);
            uint4 rg = *reinterpret_cast<const uint4 *>(dO + hb + tq * D + m * 32 + g4 * 8);
            if (c16 >= Gw) { rq = make_uint4(0u, 0u, 0u, 0u); rg = rq; }
            qa[m] = __builtin_bit_cast(bf16x8_t, rq);
            ga[m] = __builtin_bit_cast(bf16x8_t, rg);
        }
    }
    // D0[q] = dO_q . O_q (stored, rounded O): lanes across the channels, then a wave reduction
#pragma unroll 1
    for (int q = 0; q < Gw; ++q) {
        const int64_t t = member_token(gm, g, mb + q);
        const uint32_t go = reinterpret_cast<const uint32_t *>(dO + hb + t * D)[lane];
        const uint32_t oo = reinterpret_cast<const uint32_t *>(O + hb + t * D)[lane];
        float d = __uint_as_float(go << 16) * __uint_as_float(oo << 16) +
                  __uint_as_float(go & 0xFFFF0000u) * __uint_as_float(oo & 0xFFFF0000u);
        d = half_sum(d);
        d += __shfl_xor(d, 32);
        if (lane == 0) q_s[q] = d;
    }
    wave_sync();
    // softmax-side state of the lanes that hold real query rows after the 16-row products: queries 4 g4 + v, g4 < 2
    float lse2[4], d0[4], dl[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const int q = 4 * (g4 & 1) + v;
        lse2[v] = q < Gw ? lse[(int64_t)bh * L + member_token(gm, g, mb + q)] * kLog2e : 0.f;
        d0[v] = q < Gw ? q_s[q] : 0.f;
        dl[v] = 0.f;
    }
    floatx16_t acc2[NC];  // acc2[nb][4 part + i]: query 4 half + i, channel 32 nb + n; parts: C head, C tail, B head, B tail
#pragma unroll
    for (int nb = 0; nb < NC; ++nb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc2[nb][i] = 0.f;
    const float c2 = scale * kLog2e;
    // this lane's addresses for the transposing reads of K (second product): rows dq_key(s, half, c16 / 4) and
    // dq_key(s, half, 4 + c16 / 4), channels 16 (g4 % 2) + 4 (c16 % 4) .. + 3 of a 32-channel block
    int kt[2][2];
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
        for (int r = 0; r < 2; ++r) kt[s][r] = dq_key(s, half, 4 * r + (c16 >> 2)) * kVRow + (g4 & 1) * 32 + (c16 & 3) * 8;

    // rows loaded whole and parked in LDS, software-pipelined, as in the forward
    constexpr int NI = 8 / NSUB;                 // load instructions (4 rows each) of this wave per tile and matrix
    const int i0 = NSUB == 1 ? 0 : NI * wave;
    int32_t jr[NI];
    bf16x8_t kr[NI], vr[NI];
    auto load_idx = [&](int t0) {
#pragma unroll
        for (int i = 0; i < NI; ++i) jr[i] = row[min(t0 + g4 + 4 * (i0 + i), te - 1)];
    };
    auto load_rows = [&]() {
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            kr[i] = *reinterpret_cast<const bf16x8_t *>(Kh + (int64_t)jr[i] * D + c16 * 8);
            vr[i] = *reinterpret_cast<const bf16x8_t *>(Vh + (int64_t)jr[i] * D + c16 * 8);
        }
    };
    if (tb < te) {
        load_idx(tb);
        load_rows();
        if (tb + 32 < te) load_idx(tb + 32);
    }
    for (int t0 = tb; t0 < te; t0 += 32) {
        const int nvalid = min(32, te - t0);
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            *reinterpret_cast<bf16x8_t *>(K_s + (g4 + 4 * (i0 + i)) * kVRow + c16 * 16) = kr[i];
            *reinterpret_cast<bf16x8_t *>(V_s + (g4 + 4 * (i0 + i)) * kVRow + c16 * 16) = vr[i];
        }
        block_sync();
        if (t0 + 32 < te) {  // wave-uniform
            load_rows();
            if (t0 + 64 < te) load_idx(t0 + 64);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {  // keys 16 s + c16
            floatx4_t as = {0.f, 0.f, 0.f, 0.f}, ap = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const bf16x8_t kb = *reinterpret_cast<const bf16x8_t *>(K_s + (16 * s + c16) * kVRow + (m * 32 + g4 * 8) * 2);
                const bf16x8_t vb = *reinterpret_cast<const bf16x8_t *>(V_s + (16 * s + c16) * kVRow + (m * 32 + g4 * 8) * 2);
                as = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qa[m], kb, as, 0, 0, 0);
                ap = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ga[m], vb, ap, 0, 0, 0);
            }
            if (g4 < 2) {  // the half-wave with the real query rows
                const int key = 16 * s + c16;
                const int ws = w_slot(key);
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float pp = key < nvalid ? fast_exp2(as[v] * c2 - lse2[v]) : 0.f;
                    dl[v] = fmaf(pp, ap[v], dl[v]);
                    const float wc = pp * (ap[v] - d0[v]);
                    uint16_t hi, lo;
                    const int r = 4 * g4 + v;
                    split_bf16(wc, hi, lo);
                    reinterpret_cast<u16_alias *>(W_s)[r * 32 + ws] = hi;
                    reinterpret_cast<u16_alias *>(W_s)[(8 + r) * 32 + ws] = lo;
                    split_bf16(pp, hi, lo);
                    reinterpret_cast<u16_alias *>(W_s)[(16 + r) * 32 + ws] = hi;
                    reinterpret_cast<u16_alias *>(W_s)[(24 + r) * 32 + ws] = lo;
                }
            }
        }
        wave_sync();
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            const bf16x8_t wa = __builtin_bit_cast(bf16x8_t, *reinterpret_cast<const uint4 *>(const_cast<const uint32_t *>(W_s) + n * 16 + s * 8 + half * 4));
#pragma unroll
            for (int nb = 0; nb < NC; ++nb)
                acc2[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wa, tr_frag(K_s + kt[s][0] + nb * 64, K_s + kt[s][1] + nb * 64), acc2[nb], 0, 0, 0);
        }
        block_sync();  // the next tile overwrites the parked rows and W_s
    }
    if (!active) return;
    // Delta of query 4 g4 + v: sum over the 16 lanes of the row group (both key sub-tiles are already in dl)
    float dt[4];
#pragma unroll
    for (int v = 0; v < 4; ++v) dt[v] = row16_sum(dl[v]);
    if (g4 < 2 && c16 == 0) {
#pragma unroll
        for (int v = 0; v < 4; ++v) q_s[8 + 4 * g4 + v] = dt[v];
    }
    wave_sync();
    if (SPLIT) {
        if (lane < Gw) pdelta[((int64_t)bh * L + member_token(gm, g, mb + lane)) * pl.S + range] = q_s[8 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int q = 4 * half + i;
            if (q < Gw) {
                const int64_t slot_id = ((int64_t)bh * L + member_token(gm, g, mb + q)) * pl.S + range;
#pragma unroll
                for (int nb = 0; nb < NC; ++nb) {
                    pa[slot_id * D + nb * 32 + n] = acc2[nb][i] + acc2[nb][4 + i];
                    pb[slot_id * D + nb * 32 + n] = acc2[nb][8 + i] + acc2[nb][12 + i];
                }
            }
        }
        return;
    }
    if (lane < Gw) delta_out[(int64_t)bh * L + member_token(gm, g, mb + lane)] = q_s[8 + lane];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = 4 * half + i;
        if (q < Gw) {
            const float dd = q_s[8 + q] - q_s[q];
            bf16_t *qrow = dQ + hb + member_token(gm, g, mb + q) * D;
#pragma unroll
            for (int nb = 0; nb < NC; ++nb) {
                const float cc = acc2[nb][i] + acc2[nb][4 + i], bb = acc2[nb][8 + i] + acc2[nb][12 + i];
                qrow[nb * 32 + n] = f32_to_bf16(scale * (cc - dd * bb));
            }
        }
    }
}

// ------------------------------------------------------------------------------------ host
GroupGeom make_group_geom(const dsv_grouping &gr)
{
    GroupGeom gm;
    gm.F = gr.F; gm.Hh = gr.Hh; gm.Ww = gr.Ww;
    gm.gf = gr.gf; gm.gh = gr.gh; gm.gw = gr.gw;
    gm.nh = gr.Hh / gr.gh; gm.nw = gr.Ww / gr.gw;
    gm.G = gr.gf * gr.gh * gr.gw;
    return gm;
}

int group_centre(const dsv_grouping &gr) { return ((gr.gf / 2) * gr.gh + gr.gh / 2) * gr.gw + gr.gw / 2; }

template <typename T, int MODE>
static dsv_status group_rows_t(const dsv_problem &p, const GroupGeom &gm, int centre, const void *in, void *out, int n_out,
                               hipStream_t st)
{
    const int64_t pieces = (int64_t)n_out * (p.d * (int)sizeof(T) / 16);
    dim3 grid((unsigned)((pieces + 255) / 256), p.B * p.H);
    hipLaunchKernelGGL((group_rows_kernel<T, MODE>), grid, dim3(256), 0, st, (const T *)in, (T *)out, p.L, p.d, n_out, gm, centre);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_group_rows(const dsv_problem &p, const dsv_grouping &gr, int mode, const void *in, void *out,
                             hipStream_t st)
{
    const GroupGeom gm = make_group_geom(gr);
    const int centre = group_centre(gr);
    const int n_out = mode == 0 ? p.L / gm.G : p.L;
    if (p.dtype == DSV_BF16) {
        if (mode == 0) return group_rows_t<bf16_t, 0>(p, gm, centre, in, out, n_out, st);
        if (mode == 1) return group_rows_t<bf16_t, 1>(p, gm, centre, in, out, n_out, st);
        return group_rows_t<bf16_t, 2>(p, gm, centre, in, out, n_out, st);
    }
    if (mode == 0) return group_rows_t<float, 0>(p, gm, centre, in, out, n_out, st);
    if (mode == 1) return group_rows_t<float, 1>(p, gm, centre, in, out, n_out, st);
    return group_rows_t<float, 2>(p, gm, centre, in, out, n_out, st);
}

dsv_status launch_group_scalar(const dsv_problem &p, const dsv_grouping &gr, const float *in, float *out, hipStream_t st,
                               bool inverse)
{
    hipLaunchKernelGGL(group_scalar_kernel, dim3((p.L + 255) / 256, p.B * p.H), dim3(256), 0, st, in, out, p.L,
                       make_group_geom(gr), inverse ? 1 : 0);
    DSV_LAUNCH_CHECK();
    return DSV_OK;
}

dsv_status launch_group_expand(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                               const int32_t *idx_g, const int32_t *idx_t_g, const int64_t *col, int32_t *idx_x,
                               int32_t *idx_t_x, int64_t *col_x, hipStream_t st)
{
    const GroupGeom gm = make_group_geom(gr);
    const int Lq = p.L / gm.G;
    for (int t = 0; t < n_tabs; ++t) {
        if (idx_x)
            hipLaunchKernelGGL(expand_idx_kernel, dim3(std::min(Lq, 8192), tabs[t].n), dim3(256), 0, st, idx_g, idx_x, Lq, gm.G, tabs[t]);
        if (idx_t_x)
            hipLaunchKernelGGL(expand_idx_t_kernel, dim3(8192, tabs[t].n), dim3(256), 0, st, idx_t_g, idx_t_x, Lq, gm.G, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    if (col_x) {
        const int64_t n = (int64_t)p.B * p.H * (p.L + 1);
        hipLaunchKernelGGL(scale_col_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, col, col_x, n, gm.G);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

// tabs: built for L rows per head (the per-query index).
dsv_status launch_group_overlap(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                                const int32_t *idx, unsigned long long *count, float *overlap, hipStream_t st)
{
    const size_t lds = (size_t)((p.L + 31) / 32) * 4;
    if (lds > (64u << 10)) return DSV_EUNSUPPORTED;
    const GroupGeom gm = make_group_geom(gr);
    const int nbh = p.B * p.H;
    hipLaunchKernelGGL(group_overlap_reset_kernel, dim3((nbh + 255) / 256), dim3(256), 0, st, count, nbh);
    DSV_LAUNCH_CHECK();
    const int Lq = p.L / gm.G;
    for (int t = 0; t < n_tabs; ++t) {
        hipLaunchKernelGGL(group_overlap_kernel, dim3(std::min(Lq, 2048), tabs[t].n), dim3(256), lds, st, idx, p.L, tabs[t], gm,
                           group_centre(gr), count);
        hipLaunchKernelGGL(group_overlap_finish_kernel, dim3(1), dim3(kMaxSlots), 0, st, count, overlap, p.L, tabs[t]);
        DSV_LAUNCH_CHECK();
    }
    return DSV_OK;
}

// Launch shapes of the group kernels: groups of at most 8 queries, four to a block (one wave each); groups of up to 16
// (32), one to a block of two (four) waves that share the parked rows.
static int groups_per_block(int G) { return G <= 8 ? 4 : 1; }
static int waves_per_group(int G) { return G <= 8 ? 1 : (G <= 16 ? 2 : 4); }

template <bool SPLIT, typename... Args>
static void launch_fwd_variant(int nsub, dim3 grid, hipStream_t st, Args... args)
{
    if (nsub == 1) hipLaunchKernelGGL((grouped_fwd_kernel<128, SPLIT, 1>), grid, dim3(256), 0, st, args...);
    else if (nsub == 2) hipLaunchKernelGGL((grouped_fwd_kernel<128, SPLIT, 2>), grid, dim3(128), 0, st, args...);
    else hipLaunchKernelGGL((grouped_fwd_kernel<128, SPLIT, 4>), grid, dim3(256), 0, st, args...);
}
template <bool SPLIT, typename... Args>
static void launch_dq_variant(int nsub, dim3 grid, hipStream_t st, Args... args)
{
    if (nsub == 1) hipLaunchKernelGGL((grouped_dq_kernel<128, SPLIT, 1>), grid, dim3(256), 0, st, args...);
    else if (nsub == 2) hipLaunchKernelGGL((grouped_dq_kernel<128, SPLIT, 2>), grid, dim3(128), 0, st, args...);
    else hipLaunchKernelGGL((grouped_dq_kernel<128, SPLIT, 4>), grid, dim3(256), 0, st, args...);
}

dsv_status launch_grouped_fwd(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                              const void *Q, const void *K, const void *V, const int32_t *idx_g, void *O, float *lse,
                              const GroupedSplit *split, hipStream_t st)
{
    if (p.dtype != DSV_BF16 || p.d != 128) return DSV_EUNSUPPORTED;
    const GroupGeom gm = make_group_geom(gr);
    if (gm.G > 32) return DSV_EUNSUPPORTED;
    const int Lq = p.L / gm.G;
    const int gpb = groups_per_block(gm.G), nsub = waves_per_group(gm.G);
    const int nqb = (Lq + gpb - 1) / gpb;
    if (!split) {
        KernelSpan span(DSV_KERNEL_FWD_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            dim3 grid(nqb, tabs[t].n);
            launch_fwd_variant<false>(nsub, grid, st, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, idx_g, (bf16_t *)O, lse,
                                      (const int32_t *)nullptr, (float *)nullptr, (float *)nullptr, (float *)nullptr, p.L, Lq,
                                      p.scale, tabs[t], gm, SplitPlan{});
            DSV_LAUNCH_CHECK();
        }
        return DSV_OK;
    }
    SplitPlan pl = split->plan;
    pl.nqb = nqb;
    dsv_status rc = launch_row_segments(p, Lq, tabs, n_tabs, pl, idx_g, split->seg, st);
    if (rc != DSV_OK) return rc;
    {
        KernelSpan span(DSV_KERNEL_FWD_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            const int64_t blocks = (int64_t)tabs[t].n * pl.S_pad * pl.nqb;
            if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
            dim3 grid((unsigned)blocks);
            launch_fwd_variant<true>(nsub, grid, st, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, idx_g, (bf16_t *)O, lse,
                                     (const int32_t *)split->seg, split->pa, split->pb, split->pc, p.L, Lq, p.scale, tabs[t], gm,
                                     pl);
            DSV_LAUNCH_CHECK();
        }
    }
    return launch_fwd_merge_bf16_128(p, split->pa, split->pb, split->pc, O, lse, pl.S, st);
}

dsv_status launch_grouped_dq(const dsv_problem &p, const dsv_grouping &gr, const HeadTable *tabs, int n_tabs,
                             const void *Q, const void *K, const void *V, const int32_t *idx_g, const void *O,
                             const float *lse, const void *dO, void *dQ, float *delta, const GroupedSplit *split,
                             hipStream_t st)
{
    if (p.dtype != DSV_BF16 || p.d != 128) return DSV_EUNSUPPORTED;
    const GroupGeom gm = make_group_geom(gr);
    if (gm.G > 32) return DSV_EUNSUPPORTED;
    const int Lq = p.L / gm.G;
    const int gpb = groups_per_block(gm.G), nsub = waves_per_group(gm.G);
    const int nqb = (Lq + gpb - 1) / gpb;
    if (!split) {
        KernelSpan span(DSV_KERNEL_DQ_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            dim3 grid(nqb, tabs[t].n);
            launch_dq_variant<false>(nsub, grid, st, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, idx_g, (const bf16_t *)O, lse,
                                     (const bf16_t *)dO, (bf16_t *)dQ, delta, (const int32_t *)nullptr, (float *)nullptr,
                                     (float *)nullptr, (float *)nullptr, p.L, Lq, p.scale, tabs[t], gm, SplitPlan{});
            DSV_LAUNCH_CHECK();
        }
        return DSV_OK;
    }
    SplitPlan pl = split->plan;
    pl.nqb = nqb;
    dsv_status rc = launch_row_segments(p, Lq, tabs, n_tabs, pl, idx_g, split->seg, st);
    if (rc != DSV_OK) return rc;
    {
        KernelSpan span(DSV_KERNEL_DQ_SWEEP, st);
        for (int t = 0; t < n_tabs; ++t) {
            const int64_t blocks = (int64_t)tabs[t].n * pl.S_pad * pl.nqb;
            if (blocks > 0x7FFFFFFF) return DSV_EUNSUPPORTED;
            dim3 grid((unsigned)blocks);
            launch_dq_variant<true>(nsub, grid, st, (const bf16_t *)Q, (const bf16_t *)K, (const bf16_t *)V, idx_g, (const bf16_t *)O, lse,
                                    (const bf16_t *)dO, (bf16_t *)dQ, delta, (const int32_t *)split->seg, split->pa, split->pb,
                                    split->pc, p.L, Lq, p.scale, tabs[t], gm, pl);
            DSV_LAUNCH_CHECK();
        }
    }
    return launch_dq_merge_bf16_128(p, split->pa, split->pb, split->pc, O, dO, dQ, delta, pl.S, st);
}

}  // namespace dsv
