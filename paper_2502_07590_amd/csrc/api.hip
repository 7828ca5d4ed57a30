// C ABI of libdsv: argument checks, workspace layout, launch order.  All checks run on the host
// before anything is enqueued; the library never allocates device memory.
#include <algorithm>
#include <initializer_list>
#include <mutex>
#include <vector>

#include "common.h"

namespace dsv {
KernelTimer g_kernel_timer;
namespace {

bool supported_d(int d) { return d == 64 || d == 128; }
bool supported_r(int r) { return r == 16 || r == 32 || r == 64; }
bool supported_dtype(int t) { return t == DSV_F32 || t == DSV_BF16; }
size_t esize(int dtype) { return dtype == DSV_BF16 ? 2 : 4; }
bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// true when every pointer is non-null and 16-byte aligned
bool ok_ptrs(std::initializer_list<const void *> ps)
{
    for (const void *p : ps)
        if (!p || !aligned16(p)) return false;
    return true;
}

dsv_status check_problem(const dsv_problem *p, bool need_r)
{
    if (!p || !p->k_per_head) return DSV_EINVAL;
    if (p->B < 1 || p->H < 1 || p->L < 1) return DSV_EINVAL;
    // (batch, head) pairs index grid.y / grid.x of several kernels (limit 65535)
    if ((int64_t)p->B * p->H > 65535) return DSV_EINVAL;
    if (p->flags & ~DSV_FLAG_SORTED_INDEX) return DSV_EINVAL;
    if (!supported_dtype(p->dtype) || !supported_d(p->d)) return DSV_EUNSUPPORTED;
    if (need_r && !supported_r(p->r)) return DSV_EUNSUPPORTED;
    // the gather kernels address a head's [L, d] matrix with 32-bit byte offsets
    if ((uint64_t)p->L * (uint64_t)p->d * esize(p->dtype) >= (1ull << 32)) return DSV_EUNSUPPORTED;
    for (int h = 0; h < p->H; ++h)
        if (p->k_per_head[h] < 1 || p->k_per_head[h] > p->L) return DSV_EINVAL;
    return DSV_OK;
}

// Launch tables: all (b, h) pairs sorted by descending k (stable), cut into groups of kMaxSlots.
// rows: index rows per head (p.L, or the number of query groups); 0 = p.L.
std::vector<HeadTable> make_tables(const dsv_problem &p, int rows = 0)
{
    const int nbh = p.B * p.H;
    if (rows == 0) rows = p.L;
    std::vector<int64_t> off(nbh + 1, 0);
    for (int bh = 0; bh < nbh; ++bh) off[bh + 1] = off[bh] + (int64_t)rows * p.k_per_head[bh % p.H];
    std::vector<int> order(nbh);
    for (int i = 0; i < nbh; ++i) order[i] = i;
    std::stable_sort(order.begin(), order.end(),
                     [&](int a, int b) { return p.k_per_head[a % p.H] > p.k_per_head[b % p.H]; });
    std::vector<HeadTable> tabs((nbh + kMaxSlots - 1) / kMaxSlots);
    for (int i = 0; i < nbh; ++i) {
        HeadTable &t = tabs[i / kMaxSlots];
        const int s = i % kMaxSlots;
        t.n = s + 1;
        t.bh[s] = order[i];
        t.k[s] = p.k_per_head[order[i] % p.H];
        t.off[s] = off[order[i]];
    }
    return tabs;
}

size_t total_pairs(const dsv_problem &p)
{
    size_t nnz = 0;
    for (int bh = 0; bh < p.B * p.H; ++bh) nnz += (size_t)p.L * p.k_per_head[bh % p.H];
    return nnz;
}

dsv_status check_workspace(const void *ws, size_t have, size_t need)
{
    if (need == 0) return DSV_OK;
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255u) || have < need) return DSV_EWORKSPACE;
    return DSV_OK;
}

// ---- workspace layouts (byte offsets, every block aligned to 256) ------------------------------
struct Stage1Layout {
    size_t qlr, klr, prefix, krem, win, todo, jcut, cnt, tflag, qc, total;
};

// transposed: also room for jcut and the per-key list lengths of the key-major emission.
// Lq: scored query rows per head (p.L, or one centre query per group: then also room for those rows, qc).
Stage1Layout stage1_layout(const dsv_problem &p, bool transposed, int Lq = 0)
{
    const bool grouped = Lq != 0;
    if (!grouped) Lq = p.L;
    const size_t nbh = (size_t)p.B * p.H;
    const size_t qp = nbh * ((Lq + 31) / 32 * 32);  // per-query state rows are padded to tiles
    Stage1Layout w{};
    size_t o = 0;
    w.qlr = o; o = align_up(o + nbh * Lq * p.r * esize(p.dtype), 256);
    w.klr = o; o = align_up(o + nbh * p.L * p.r * esize(p.dtype), 256);
    w.prefix = o; o = align_up(o + qp * 4, 256);
    w.krem = o; o = align_up(o + qp * 4, 256);
    w.win = o; o = align_up(o + qp * 4, 256);
    w.todo = o; o = align_up(o + (1 + nbh * ((Lq + 31) / 32)) * 4, 256);
    w.jcut = o; if (transposed) o = align_up(o + qp * 4, 256);
    w.cnt = o; if (transposed) o = align_up(o + nbh * p.L * 4, 256);
    w.tflag = o; if (transposed) o = align_up(o + nbh * ((Lq + 31) / 32) * 4, 256);
    w.qc = o; if (grouped) o = align_up(o + nbh * Lq * p.d * esize(p.dtype), 256);
    w.total = o;
    return w;
}

// Cubes must tile the grid, and the grid must be the problem's L tokens.
dsv_status check_grouping(const dsv_problem &p, const dsv_grouping *g)
{
    if (!g) return DSV_EINVAL;
    if (g->F < 1 || g->Hh < 1 || g->Ww < 1 || g->gf < 1 || g->gh < 1 || g->gw < 1) return DSV_EINVAL;
    if ((int64_t)g->F * g->Hh * g->Ww != (int64_t)p.L) return DSV_EINVAL;
    if (g->F % g->gf || g->Hh % g->gh || g->Ww % g->gw) return DSV_EINVAL;
    if ((int64_t)g->gf * g->gh * g->gw > 64) return DSV_EUNSUPPORTED;
    return DSV_OK;
}
int group_size(const dsv_grouping &g) { return g.gf * g.gh * g.gw; }

// Whether stage 2 runs its L2-blocked kernels: sorted indices promised and more than one range.
bool use_split(const dsv_problem &p, const SplitPlan &pl) { return (p.flags & DSV_FLAG_SORTED_INDEX) && pl.S > 1; }

struct FwdLayout {
    bool split;
    SplitPlan plan;
    size_t seg, pm, pl, pacc, hist, order, total;
};

FwdLayout fwd_layout(const dsv_problem &p)
{
    FwdLayout w{};
    w.plan = make_split_plan(p, kFwdRangeBytes);
    w.split = use_split(p, w.plan);
    if (!w.split) return w;
    const size_t rows = (size_t)p.B * p.H * p.L;
    size_t o = 0;
    w.seg = o; o = align_up(o + rows * (w.plan.S + 1) * 4, 256);
    w.pm = o; o = align_up(o + rows * w.plan.S * 4, 256);
    w.pl = o; o = align_up(o + rows * w.plan.S * 4, 256);
    w.pacc = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
    w.hist = o; o = align_up(o + (size_t)p.B * p.H * w.plan.S * ((size_t)w.plan.range_len + 1) * 4, 256);
    w.order = o; o = align_up(o + rows * w.plan.S * 4, 256);
    w.total = o;
    return w;
}

// One split backward step (dq or dkdv): segment pointers and two [rows, S, d] partial arrays
// (+ [rows, S] for the dq step's Delta partials; laid out for both so that the steps can share it).
struct StepLayout {
    bool split;
    SplitPlan plan;
    size_t seg, pa, pb, pdelta, hist, order, rowstat, total;
};

StepLayout step_layout(const dsv_problem &p)
{
    StepLayout w{};
    w.plan = make_split_plan(p, kBwdRangeBytes);
    w.split = use_split(p, w.plan);
    if (!w.split) return w;
    const size_t nbh = (size_t)p.B * p.H;
    const size_t rows = nbh * p.L;
    size_t o = 0;
    w.seg = o; o = align_up(o + rows * (w.plan.S + 1) * 4, 256);
    w.pa = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
    w.pb = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
    w.pdelta = o; o = align_up(o + rows * w.plan.S * 4, 256);
    w.hist = o; o = align_up(o + nbh * w.plan.S * ((size_t)w.plan.range_len + 1) * 4, 256);
    w.order = o; o = align_up(o + rows * w.plan.S * 4, 256);
    w.rowstat = o; o = align_up(o + rows * 8, 256);
    w.total = o;
    return w;
}

BwdSplitWorkspace step_buffers(char *ws, const StepLayout &w)
{
    BwdSplitWorkspace b;
    b.seg = reinterpret_cast<int32_t *>(ws + w.seg);
    b.pa = reinterpret_cast<float *>(ws + w.pa);
    b.pb = reinterpret_cast<float *>(ws + w.pb);
    b.pdelta = reinterpret_cast<float *>(ws + w.pdelta);
    b.hist = reinterpret_cast<int32_t *>(ws + w.hist);
    b.order = reinterpret_cast<int32_t *>(ws + w.order);
    b.rowstat = reinterpret_cast<float2 *>(ws + w.rowstat);
    return b;
}

// Whole backward.  own_transpose: the call builds the key-major index itself (dsv_sparse_attn_bwd);
// otherwise the caller brings it (dsv_sparse_attn_bwd_t).
struct BwdLayout {
    size_t delta, cnt, cnt_bytes, col, idxT, step, step_bytes, total;
};

BwdLayout bwd_layout(const dsv_problem &p, bool own_transpose)
{
    const size_t nbh = (size_t)p.B * p.H;
    const size_t tok = nbh * p.L;
    BwdLayout w{};
    size_t o = 0;
    w.delta = o; o = align_up(o + tok * 4, 256);
    if (own_transpose) {
        w.cnt = o; w.cnt_bytes = idx_transpose_bytes(p); o += w.cnt_bytes;
        w.col = o; o = align_up(o + nbh * ((size_t)p.L + 1) * 8, 256);
        w.idxT = o; o = align_up(o + total_pairs(p) * 4, 256);
    }
    // own_transpose: the lists come out ascending, so the dkdv step runs the L2-blocked kernel whatever p.flags says
    dsv_problem sorted = p;
    sorted.flags |= DSV_FLAG_SORTED_INDEX;
    w.step = o; w.step_bytes = own_transpose ? std::max(step_layout(p).total, step_layout(sorted).total) : step_layout(p).total;
    o += w.step_bytes;
    w.total = o;
    return w;
}

}  // namespace
}  // namespace dsv

using namespace dsv;

// ---- scratch of dsv_lowrank_topk_noalloc ---------------------------------------------------------
// A fixed array in the library's device image: every GPU that loads the library holds its own copy at
// its own address.  In host code the array's NAME is only a handle for hipGetSymbolAddress -- it is not
// a device address and is never passed to a kernel, a copy or a fill; the address is looked up once
// per device (with that device current) and kept here.
constexpr size_t kNoallocBytes = 32u << 20;
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void *g_scratch_ptr[kMaxDevices] = {};

// Device address of this GPU's copy of `scratch`; nullptr (and *err set) on failure.
static void *noalloc_scratch(dsv_status *err)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { *err = DSV_EHIP; return nullptr; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { *err = DSV_EHIP; return nullptr; }
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

extern "C" {

const char *dsv_version(void) { return "dsv 0.4 (gfx950)"; }

const char *dsv_status_string(dsv_status s)
{
    switch (s) {
    case DSV_OK: return "ok";
    case DSV_EINVAL: return "invalid argument";
    case DSV_EUNSUPPORTED: return "unsupported head dimension, rank or dtype";
    case DSV_EWORKSPACE: return "workspace missing, misaligned or too small";
    case DSV_EHIP: return "HIP runtime error";
    default: return "unknown status";
    }
}

dsv_status dsv_idx_offsets(const dsv_problem *p, int64_t *off)
{
    if (!p || !p->k_per_head || !off || p->B < 1 || p->H < 1 || p->L < 1) return DSV_EINVAL;
    for (int h = 0; h < p->H; ++h)
        if (p->k_per_head[h] < 1 || p->k_per_head[h] > p->L) return DSV_EINVAL;
    off[0] = 0;
    for (int bh = 0; bh < p->B * p->H; ++bh) off[bh + 1] = off[bh] + (int64_t)p->L * p->k_per_head[bh % p->H];
    return DSV_OK;
}

// ------------------------------------------------------------------------------------ stage 1
// grp == nullptr: every query is scored; else only the centre query of every group (idx, idx_t then hold
// one row per group and lists of groups).
static dsv_status lowrank_topk_impl(const dsv_problem *p, const dsv_grouping *grp, const void *Q, const void *K,
                                    const void *Wq, const void *Wk, int32_t *idx, int32_t *idx_t, int64_t *col_ptr,
                                    bool transposed, void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, true);
    if (st != DSV_OK) return st;
    if (grp && (st = check_grouping(*p, grp)) != DSV_OK) return st;
    if (!ok_ptrs({Q, K, Wq, Wk, idx})) return DSV_EINVAL;
    if (transposed && !ok_ptrs({idx_t, col_ptr})) return DSV_EINVAL;
    const int Lq = grp ? p->L / group_size(*grp) : p->L;
    const Stage1Layout w = stage1_layout(*p, transposed, grp ? Lq : 0);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    char *ws = static_cast<char *>(workspace);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const void *Qsrc = Q;
    if (grp) {
        st = launch_group_rows(*p, *grp, 0, Q, ws + w.qc, stream);
        if (st != DSV_OK) return st;
        Qsrc = ws + w.qc;
    }
    st = launch_project(*p, Lq, Qsrc, K, Wq, Wk, ws + w.qlr, ws + w.klr, stream);
    if (st != DSV_OK) return st;
    SelectBuffers b;
    b.prefix = reinterpret_cast<uint32_t *>(ws + w.prefix);
    b.krem = reinterpret_cast<int32_t *>(ws + w.krem);
    b.win = reinterpret_cast<uint32_t *>(ws + w.win);
    b.todo = reinterpret_cast<int32_t *>(ws + w.todo);
    b.idx = idx;
    b.jcut = transposed ? reinterpret_cast<int32_t *>(ws + w.jcut) : nullptr;
    b.cnt = transposed ? reinterpret_cast<int32_t *>(ws + w.cnt) : nullptr;
    b.tile_flag = transposed ? reinterpret_cast<int32_t *>(ws + w.tflag) : nullptr;
    b.col = transposed ? col_ptr : nullptr;
    b.idx_t = transposed ? idx_t : nullptr;
    const std::vector<HeadTable> tabs = make_tables(*p, Lq);
    return launch_select(*p, Lq, tabs.data(), (int)tabs.size(), ws + w.qlr, ws + w.klr, b, stream);
}

size_t dsv_lowrank_topk_workspace(const dsv_problem *p)
{
    if (check_problem(p, true) != DSV_OK) return 0;
    return stage1_layout(*p, false).total;
}

dsv_status dsv_lowrank_topk(const dsv_problem *p, const void *Q, const void *K, const void *Wq, const void *Wk,
                            int32_t *idx, void *workspace, size_t ws_bytes, void *hip_stream)
{
    return lowrank_topk_impl(p, nullptr, Q, K, Wq, Wk, idx, nullptr, nullptr, false, workspace, ws_bytes, hip_stream);
}

size_t dsv_lowrank_topk_noalloc_max_bytes(void) { return kNoallocBytes; }

dsv_status dsv_lowrank_topk_noalloc(const dsv_problem *p, const void *Q, const void *K, const void *Wq, const void *Wk,
                                    int32_t *idx, void *hip_stream)
{
    // everything that can be refused is refused before the scratch is looked up
    dsv_status st = check_problem(p, true);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({Q, K, Wq, Wk, idx})) return DSV_EINVAL;
    const size_t need = stage1_layout(*p, false).total;
    if (need > kNoallocBytes) return DSV_EWORKSPACE;
    void *ws = noalloc_scratch(&st);
    if (!ws) return st;
    // every buffer of the layout is written by the kernels of this call before it is read (projections by
    // project_kernel, thresholds and tie budgets by the first radix pass), so what an earlier call left in
    // the array does not matter
    return lowrank_topk_impl(p, nullptr, Q, K, Wq, Wk, idx, nullptr, nullptr, false, ws, kNoallocBytes, hip_stream);
}

size_t dsv_lowrank_topk_t_workspace(const dsv_problem *p)
{
    if (check_problem(p, true) != DSV_OK) return 0;
    return stage1_layout(*p, true).total;
}

dsv_status dsv_lowrank_topk_t(const dsv_problem *p, const void *Q, const void *K, const void *Wq, const void *Wk,
                              int32_t *idx, int32_t *idx_t, int64_t *col_ptr, void *workspace, size_t ws_bytes,
                              void *hip_stream)
{
    return lowrank_topk_impl(p, nullptr, Q, K, Wq, Wk, idx, idx_t, col_ptr, true, workspace, ws_bytes, hip_stream);
}

// ------------------------------------------------------------------------------------ stage 2 forward
size_t dsv_sparse_attn_fwd_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return fwd_layout(*p).total;
}

dsv_status dsv_sparse_attn_fwd(const dsv_problem *p, const void *Q, const void *K, const void *V, const int32_t *idx,
                               void *O, float *lse, void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({Q, K, V, idx, O, lse})) return DSV_EINVAL;
    const FwdLayout w = fwd_layout(*p);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!w.split) return launch_sparse_fwd(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx, O, lse, stream);
    char *ws = static_cast<char *>(workspace);
    FwdSplitWorkspace b;
    b.seg = reinterpret_cast<int32_t *>(ws + w.seg);
    b.pm = reinterpret_cast<float *>(ws + w.pm);
    b.pl = reinterpret_cast<float *>(ws + w.pl);
    b.pacc = reinterpret_cast<float *>(ws + w.pacc);
    b.hist = reinterpret_cast<int32_t *>(ws + w.hist);
    b.order = reinterpret_cast<int32_t *>(ws + w.order);
    return launch_sparse_fwd_split(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx, O, lse, w.plan, b, stream);
}

// ------------------------------------------------------------------------------------ stage 2 backward
size_t dsv_sparse_attn_bwd_dq_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return step_layout(*p).total;
}

dsv_status dsv_sparse_attn_bwd_dq(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                  const int32_t *idx, const void *O, const float *lse, const void *dO, void *dQ,
                                  float *delta, void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({Q, K, V, idx, O, lse, dO, dQ, delta})) return DSV_EINVAL;
    const StepLayout w = step_layout(*p);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!w.split) return launch_bwd_dq(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx, O, lse, dO, dQ, delta, stream);
    return launch_bwd_dq_split(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx, O, lse, dO, dQ, delta, w.plan,
                               step_buffers(static_cast<char *>(workspace), w), stream);
}

size_t dsv_idx_transpose_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return idx_transpose_bytes(*p);
}

dsv_status dsv_idx_transpose(const dsv_problem *p, const int32_t *idx, int32_t *idx_t, int64_t *col_ptr,
                             void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({idx, idx_t, col_ptr})) return DSV_EINVAL;
    const size_t need = dsv_idx_transpose_workspace(p);
    st = check_workspace(workspace, ws_bytes, need);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    return launch_idx_transpose(*p, tabs.data(), (int)tabs.size(), idx, idx_t, col_ptr,
                                static_cast<int32_t *>(workspace), need, static_cast<hipStream_t>(hip_stream));
}

size_t dsv_sparse_attn_bwd_dkdv_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return step_layout(*p).total;
}

dsv_status dsv_sparse_attn_bwd_dkdv(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                    const int32_t *idx_t, const int64_t *col_ptr, const float *lse, const float *delta,
                                    const void *dO, void *dK, void *dV, void *workspace, size_t ws_bytes,
                                    void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({Q, K, V, idx_t, col_ptr, lse, delta, dO, dK, dV})) return DSV_EINVAL;
    const StepLayout w = step_layout(*p);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (!w.split)
        return launch_bwd_dkdv(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx_t, col_ptr, lse, delta, dO, dK, dV,
                               stream);
    return launch_bwd_dkdv_split(*p, tabs.data(), (int)tabs.size(), Q, K, V, idx_t, col_ptr, lse, delta, dO, dK, dV,
                                 w.plan, step_buffers(static_cast<char *>(workspace), w), stream);
}

size_t dsv_sparse_attn_bwd_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return bwd_layout(*p, true).total;
}

dsv_status dsv_sparse_attn_bwd(const dsv_problem *p, const void *Q, const void *K, const void *V, const int32_t *idx,
                               const void *O, const float *lse, const void *dO, void *dQ, void *dK, void *dV,
                               void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({O, dQ, dK, dV})) return DSV_EINVAL;
    const BwdLayout w = bwd_layout(*p, true);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    char *ws = static_cast<char *>(workspace);
    float *delta = reinterpret_cast<float *>(ws + w.delta);
    int64_t *col = reinterpret_cast<int64_t *>(ws + w.col);
    int32_t *idx_t = reinterpret_cast<int32_t *>(ws + w.idxT);
    st = dsv_sparse_attn_bwd_dq(p, Q, K, V, idx, O, lse, dO, dQ, delta, ws + w.step, w.step_bytes, hip_stream);
    if (st != DSV_OK) return st;
    st = dsv_idx_transpose(p, idx, idx_t, col, ws + w.cnt, w.cnt_bytes, hip_stream);
    if (st != DSV_OK) return st;
    // the lists built here are ascending in the query index whatever the order inside the rows of idx is: the dkdv
    // step may run the L2-blocked kernel
    dsv_problem sorted = *p;
    sorted.flags |= DSV_FLAG_SORTED_INDEX;
    return dsv_sparse_attn_bwd_dkdv(&sorted, Q, K, V, idx_t, col, lse, delta, dO, dK, dV, ws + w.step, w.step_bytes, hip_stream);
}

size_t dsv_sparse_attn_bwd_t_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return bwd_layout(*p, false).total;
}

dsv_status dsv_sparse_attn_bwd_t(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                 const int32_t *idx, const int32_t *idx_t, const int64_t *col_ptr, const void *O,
                                 const float *lse, const void *dO, void *dQ, void *dK, void *dV, void *workspace,
                                 size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({O, dQ, dK, dV, idx_t, col_ptr})) return DSV_EINVAL;
    const BwdLayout w = bwd_layout(*p, false);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    char *ws = static_cast<char *>(workspace);
    float *delta = reinterpret_cast<float *>(ws + w.delta);
    st = dsv_sparse_attn_bwd_dq(p, Q, K, V, idx, O, lse, dO, dQ, delta, ws + w.step, w.step_bytes, hip_stream);
    if (st != DSV_OK) return st;
    return dsv_sparse_attn_bwd_dkdv(p, Q, K, V, idx_t, col_ptr, lse, delta, dO, dK, dV, ws + w.step, w.step_bytes,
                                    hip_stream);
}

// ------------------------------------------------------------------------------------ query grouping
size_t dsv_lowrank_topk_grouped_workspace(const dsv_problem *p, const dsv_grouping *g)
{
    if (check_problem(p, true) != DSV_OK || check_grouping(*p, g) != DSV_OK) return 0;
    return stage1_layout(*p, true, p->L / group_size(*g)).total;
}

dsv_status dsv_lowrank_topk_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                    const void *Wq, const void *Wk, int32_t *idx_g, int32_t *idx_t_g, int64_t *col_ptr,
                                    void *workspace, size_t ws_bytes, void *hip_stream)
{
    if (!g) return DSV_EINVAL;
    if ((idx_t_g == nullptr) != (col_ptr == nullptr)) return DSV_EINVAL;
    return lowrank_topk_impl(p, g, Q, K, Wq, Wk, idx_g, idx_t_g, col_ptr, idx_t_g != nullptr, workspace, ws_bytes,
                             hip_stream);
}

namespace {
// Scratch of one L2-blocked grouped kernel (forward or dq): segment pointers per group row and per-(token row,
// range) partials.  split == false: the plain kernels (rows in any order, or a single range), no scratch.
struct GroupedStepLayout {
    bool split;
    SplitPlan plan;
    size_t seg, pa, pb, pc, total;
};
GroupedStepLayout grouped_step_layout(const dsv_problem &p, const dsv_grouping &g, bool dq)
{
    GroupedStepLayout w{};
    w.plan = make_split_plan(p, kBwdRangeBytes);
    w.split = use_split(p, w.plan);
    if (!w.split) return w;
    const size_t nbh = (size_t)p.B * p.H, rows = nbh * p.L, Lq = p.L / group_size(g);
    size_t o = 0;
    w.seg = o; o = align_up(o + nbh * Lq * (w.plan.S + 1) * 4, 256);
    if (dq) {
        w.pa = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
        w.pb = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
        w.pc = o; o = align_up(o + rows * w.plan.S * 4, 256);
    } else {
        w.pa = o; o = align_up(o + rows * w.plan.S * 4, 256);
        w.pb = o; o = align_up(o + rows * w.plan.S * 4, 256);
        w.pc = o; o = align_up(o + rows * w.plan.S * p.d * 4, 256);
    }
    w.total = o;
    return w;
}
GroupedSplit grouped_split(char *ws, const GroupedStepLayout &w)
{
    GroupedSplit s;
    s.plan = w.plan;
    s.seg = reinterpret_cast<int32_t *>(ws + w.seg);
    s.pa = reinterpret_cast<float *>(ws + w.pa);
    s.pb = reinterpret_cast<float *>(ws + w.pb);
    s.pc = reinterpret_cast<float *>(ws + w.pc);
    return s;
}

// The group kernels proper exist for bf16, d = 128 and groups of at most 32 queries.  Every other case (fp32, d = 64,
// larger cubes) runs the per-query kernels on the queries reordered group by group, with the group index expanded to
// one row per query: the same results, without the saving.
bool grouped_native(const dsv_problem &p, const dsv_grouping &g) { return p.dtype == DSV_BF16 && p.d == 128 && group_size(g) <= 32; }

struct GroupedFwdGeneral {
    size_t qp, op, lsep, idxx, step, step_bytes, total;
};
GroupedFwdGeneral grouped_fwd_general(const dsv_problem &p)
{
    const size_t nbh = (size_t)p.B * p.H;
    const size_t rows = nbh * p.L * p.d * esize(p.dtype);
    GroupedFwdGeneral w{};
    size_t o = 0;
    w.qp = o; o = align_up(o + rows, 256);
    w.op = o; o = align_up(o + rows, 256);
    w.lsep = o; o = align_up(o + nbh * p.L * 4, 256);
    w.idxx = o; o = align_up(o + total_pairs(p) * 4, 256);
    w.step = o; w.step_bytes = fwd_layout(p).total; o += w.step_bytes;
    w.total = o;
    return w;
}

struct GroupedBwdLayout {
    bool lists_of_groups;  // the dkdv sweep reads the lists of groups as they are (no per-query copy of them)
    size_t delta, qp, gop, lsep, deltap, idxtx, colx, op, dqp, idxx, step, step_bytes, total;
};
GroupedBwdLayout grouped_bwd_layout(const dsv_problem &p, const dsv_grouping &g)
{
    const size_t nbh = (size_t)p.B * p.H;
    const size_t rows = nbh * p.L * p.d * esize(p.dtype);
    const bool native = grouped_native(p, g);
    dsv_problem sorted = p;
    sorted.flags |= DSV_FLAG_SORTED_INDEX;
    GroupedBwdLayout w{};
    // the L2-blocked sweep expands a list of groups while it stages it; the plain sweep (a single range) and the
    // general path take the per-query form written out
    w.lists_of_groups = native && step_layout(sorted).split && (uint64_t)p.L * (uint64_t)group_size(g) < (1ull << 32);
    size_t o = 0;
    w.delta = o; o = align_up(o + nbh * p.L * 4, 256);
    w.qp = o; o = align_up(o + rows, 256);
    w.gop = o; o = align_up(o + rows, 256);
    w.lsep = o; o = align_up(o + nbh * p.L * 4, 256);
    w.deltap = o; o = align_up(o + nbh * p.L * 4, 256);
    if (!w.lists_of_groups) {
        w.idxtx = o; o = align_up(o + total_pairs(p) * 4, 256);
        w.colx = o; o = align_up(o + nbh * ((size_t)p.L + 1) * 8, 256);
    }
    if (!native) {   // the per-query dq step on reordered queries: O and dQ in that order, one index row per query
        w.op = o; o = align_up(o + rows, 256);
        w.dqp = o; o = align_up(o + rows, 256);
        w.idxx = o; o = align_up(o + total_pairs(p) * 4, 256);
    }
    // the dq step's scratch and the dkdv step's are never live together
    const size_t dq_bytes = native ? grouped_step_layout(p, g, true).total : step_layout(p).total;
    w.step = o; w.step_bytes = std::max(dq_bytes, step_layout(sorted).total); o += w.step_bytes;
    w.total = o;
    return w;
}
}  // namespace

size_t dsv_sparse_attn_fwd_grouped_workspace(const dsv_problem *p, const dsv_grouping *g)
{
    if (check_problem(p, false) != DSV_OK || check_grouping(*p, g) != DSV_OK) return 0;
    return grouped_native(*p, *g) ? grouped_step_layout(*p, *g, false).total : grouped_fwd_general(*p).total;
}

dsv_status dsv_sparse_attn_fwd_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                       const void *V, const int32_t *idx_g, void *O, float *lse, void *workspace,
                                       size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if ((st = check_grouping(*p, g)) != DSV_OK) return st;
    if (!ok_ptrs({Q, K, V, idx_g, O, lse})) return DSV_EINVAL;
    if (!grouped_native(*p, *g)) {
        const GroupedFwdGeneral w = grouped_fwd_general(*p);
        st = check_workspace(workspace, ws_bytes, w.total);
        if (st != DSV_OK) return st;
        char *ws = static_cast<char *>(workspace);
        hipStream_t stream = static_cast<hipStream_t>(hip_stream);
        const std::vector<HeadTable> tabs = make_tables(*p, p->L / group_size(*g));
        int32_t *idx_x = reinterpret_cast<int32_t *>(ws + w.idxx);
        float *lsep = reinterpret_cast<float *>(ws + w.lsep);
        if ((st = launch_group_rows(*p, *g, 1, Q, ws + w.qp, stream)) != DSV_OK) return st;
        st = launch_group_expand(*p, *g, tabs.data(), (int)tabs.size(), idx_g, nullptr, nullptr, idx_x, nullptr, nullptr, stream);
        if (st != DSV_OK) return st;
        st = dsv_sparse_attn_fwd(p, ws + w.qp, K, V, idx_x, ws + w.op, lsep, w.step_bytes ? ws + w.step : nullptr, w.step_bytes,
                                 hip_stream);
        if (st != DSV_OK) return st;
        if ((st = launch_group_rows(*p, *g, 2, ws + w.op, O, stream)) != DSV_OK) return st;
        return launch_group_scalar(*p, *g, lsep, lse, stream, true);
    }
    const GroupedStepLayout w = grouped_step_layout(*p, *g, false);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p, p->L / group_size(*g));
    GroupedSplit sp;
    if (w.split) sp = grouped_split(static_cast<char *>(workspace), w);
    return launch_grouped_fwd(*p, *g, tabs.data(), (int)tabs.size(), Q, K, V, idx_g, O, lse, w.split ? &sp : nullptr,
                              static_cast<hipStream_t>(hip_stream));
}

size_t dsv_sparse_attn_bwd_grouped_workspace(const dsv_problem *p, const dsv_grouping *g)
{
    if (check_problem(p, false) != DSV_OK || check_grouping(*p, g) != DSV_OK) return 0;
    return grouped_bwd_layout(*p, *g).total;
}

dsv_status dsv_sparse_attn_bwd_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                       const void *V, const int32_t *idx_g, const int32_t *idx_t_g,
                                       const int64_t *col_ptr, const void *O, const float *lse, const void *dO, void *dQ,
                                       void *dK, void *dV, void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if ((st = check_grouping(*p, g)) != DSV_OK) return st;
    if (!ok_ptrs({Q, K, V, idx_g, idx_t_g, col_ptr, O, lse, dO, dQ, dK, dV})) return DSV_EINVAL;
    const bool native = grouped_native(*p, *g);
    const GroupedBwdLayout w = grouped_bwd_layout(*p, *g);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    char *ws = static_cast<char *>(workspace);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const std::vector<HeadTable> tabs = make_tables(*p, p->L / group_size(*g));
    float *delta = reinterpret_cast<float *>(ws + w.delta);
    float *lsep = reinterpret_cast<float *>(ws + w.lsep), *deltap = reinterpret_cast<float *>(ws + w.deltap);
    // queries reordered group by group: a group's members become neighbours, and the per-query lists that the lists of
    // groups stand for come out ascending
    if ((st = launch_group_rows(*p, *g, 1, Q, ws + w.qp, stream)) != DSV_OK) return st;
    if ((st = launch_group_rows(*p, *g, 1, dO, ws + w.gop, stream)) != DSV_OK) return st;
    if ((st = launch_group_scalar(*p, *g, lse, lsep, stream)) != DSV_OK) return st;
    if (native) {
        // dQ step, group by group (K and V rows gathered once per group)
        const GroupedStepLayout dqw = grouped_step_layout(*p, *g, true);
        GroupedSplit sp;
        if (dqw.split) sp = grouped_split(ws + w.step, dqw);
        st = launch_grouped_dq(*p, *g, tabs.data(), (int)tabs.size(), Q, K, V, idx_g, O, lse, dO, dQ, delta,
                               dqw.split ? &sp : nullptr, stream);
        if (st != DSV_OK) return st;
        if ((st = launch_group_scalar(*p, *g, delta, deltap, stream)) != DSV_OK) return st;
    } else {
        // dQ step by the per-query kernel on the reordered queries, one (expanded) index row per query
        int32_t *idx_x = reinterpret_cast<int32_t *>(ws + w.idxx);
        if ((st = launch_group_rows(*p, *g, 1, O, ws + w.op, stream)) != DSV_OK) return st;
        st = launch_group_expand(*p, *g, tabs.data(), (int)tabs.size(), idx_g, nullptr, nullptr, idx_x, nullptr, nullptr, stream);
        if (st != DSV_OK) return st;
        const size_t dq_bytes = step_layout(*p).total;
        st = dsv_sparse_attn_bwd_dq(p, ws + w.qp, K, V, idx_x, ws + w.op, lsep, ws + w.gop, ws + w.dqp, deltap,
                                    dq_bytes ? ws + w.step : nullptr, dq_bytes, hip_stream);
        if (st != DSV_OK) return st;
        if ((st = launch_group_rows(*p, *g, 2, ws + w.dqp, dQ, stream)) != DSV_OK) return st;
    }
    // dK, dV step: the per-query key-major sweep on the reordered queries
    if (w.lists_of_groups) {
        dsv_problem sorted = *p;
        sorted.flags |= DSV_FLAG_SORTED_INDEX;
        const StepLayout kw = step_layout(sorted);
        return launch_bwd_dkdv_split(sorted, tabs.data(), (int)tabs.size(), ws + w.qp, K, V, idx_t_g, col_ptr, lsep, deltap,
                                     ws + w.gop, dK, dV, kw.plan, step_buffers(ws + w.step, kw), stream, group_size(*g));
    }
    st = launch_group_expand(*p, *g, tabs.data(), (int)tabs.size(), idx_g, idx_t_g, col_ptr, nullptr,
                             reinterpret_cast<int32_t *>(ws + w.idxtx), reinterpret_cast<int64_t *>(ws + w.colx), stream);
    if (st != DSV_OK) return st;
    dsv_problem sorted = *p;
    sorted.flags |= DSV_FLAG_SORTED_INDEX;
    const size_t dkdv_bytes = step_layout(sorted).total;
    return dsv_sparse_attn_bwd_dkdv(&sorted, ws + w.qp, K, V, reinterpret_cast<int32_t *>(ws + w.idxtx),
                                    reinterpret_cast<int64_t *>(ws + w.colx), lsep, deltap, ws + w.gop, dK, dV,
                                    dkdv_bytes ? ws + w.step : nullptr, dkdv_bytes, hip_stream);
}

// ------------------------------------------------------------------------------------ group-size profiling
size_t dsv_group_overlap_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return align_up((size_t)p->B * p->H * 8, 256);
}

dsv_status dsv_group_overlap(const dsv_problem *p, const dsv_grouping *g, const int32_t *idx, float *overlap,
                             void *workspace, size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if ((st = check_grouping(*p, g)) != DSV_OK) return st;
    if (!ok_ptrs({idx, overlap})) return DSV_EINVAL;
    st = check_workspace(workspace, ws_bytes, dsv_group_overlap_workspace(p));
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    return launch_group_overlap(*p, *g, tabs.data(), (int)tabs.size(), idx, static_cast<unsigned long long *>(workspace),
                                overlap, static_cast<hipStream_t>(hip_stream));
}

size_t dsv_choose_grouping_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return dsv_group_overlap_workspace(p) + align_up((size_t)p->B * p->H * 4, 256);
}

dsv_status dsv_choose_grouping(const dsv_problem *p, int32_t F, int32_t Hh, int32_t Ww, const int32_t *cubes, int32_t n,
                               const int32_t *idx, float min_overlap, int32_t *chosen, float *overlaps, void *workspace,
                               size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!cubes || !chosen || n < 1 || !ok_ptrs({idx})) return DSV_EINVAL;
    st = check_workspace(workspace, ws_bytes, dsv_choose_grouping_workspace(p));
    if (st != DSV_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int nbh = p->B * p->H;
    float *dev = reinterpret_cast<float *>(static_cast<char *>(workspace) + dsv_group_overlap_workspace(p));
    std::vector<float> host(nbh);
    int best = -1, best_members = 0;
    for (int c = 0; c < n; ++c) {
        const dsv_grouping g{F, Hh, Ww, cubes[3 * c], cubes[3 * c + 1], cubes[3 * c + 2]};
        const dsv_status ok = check_grouping(*p, &g);
        if (ok != DSV_OK) {   // does not tile the grid (or is too large): not a candidate
            if (overlaps) for (int e = 0; e < nbh; ++e) overlaps[(size_t)c * nbh + e] = -1.f;
            continue;
        }
        st = dsv_group_overlap(p, &g, idx, dev, workspace, dsv_group_overlap_workspace(p), hip_stream);
        if (st != DSV_OK) return st;
        DSV_HIP_CHECK(hipMemcpyAsync(host.data(), dev, (size_t)nbh * 4, hipMemcpyDeviceToHost, stream));
        DSV_HIP_CHECK(hipStreamSynchronize(stream));
        bool all = true;
        for (int e = 0; e < nbh; ++e) {
            if (overlaps) overlaps[(size_t)c * nbh + e] = host[e];
            all = all && host[e] >= min_overlap;
        }
        if (all && group_size(g) > best_members) { best = c; best_members = group_size(g); }
    }
    *chosen = best;
    return DSV_OK;
}

// ------------------------------------------------------------------------------------ predictor side
size_t dsv_predictor_loss_workspace(const dsv_problem *p, int32_t n_rows)
{
    if (check_problem(p, true) != DSV_OK || n_rows < 1 || n_rows > p->L) return 0;
    return predictor_layout(*p, n_rows).total;
}

dsv_status dsv_predictor_loss(const dsv_problem *p, const void *Q, const void *K, const void *Wq, const void *Wk,
                              const int32_t *rows, int32_t n_rows, float *loss, float *dWq, float *dWk, void *workspace,
                              size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, true);
    if (st != DSV_OK) return st;
    if (n_rows < 1 || n_rows > p->L) return DSV_EINVAL;
    if (!ok_ptrs({Q, K, Wq, Wk, loss, dWq, dWk}) || !rows) return DSV_EINVAL;
    const PredictorLayout w = predictor_layout(*p, n_rows);
    st = check_workspace(workspace, ws_bytes, w.total);
    if (st != DSV_OK) return st;
    return launch_predictor_loss(*p, Q, K, Wq, Wk, rows, n_rows, loss, dWq, dWk, static_cast<char *>(workspace), w,
                                 static_cast<hipStream_t>(hip_stream));
}

size_t dsv_profile_sparsity_workspace(const dsv_problem *p, int32_t n_rows)
{
    if (check_problem(p, false) != DSV_OK || n_rows < 1 || n_rows > p->L) return 0;
    return profile_workspace_bytes(*p, n_rows);
}

dsv_status dsv_profile_sparsity(const dsv_problem *p, const void *Q, const void *K, const int32_t *rows, int32_t n_rows,
                                float mass, int32_t *counts, float *sparsity, float *ema, float alpha, void *workspace,
                                size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (n_rows < 1 || n_rows > p->L || !(mass > 0.f && mass < 1.f) || !(alpha >= 0.f && alpha <= 1.f)) return DSV_EINVAL;
    if (!ok_ptrs({Q, K}) || !rows || !counts || !sparsity) return DSV_EINVAL;
    st = check_workspace(workspace, ws_bytes, profile_workspace_bytes(*p, n_rows));
    if (st != DSV_OK) return st;
    return launch_profile_sparsity(*p, Q, K, rows, n_rows, mass, counts, sparsity, ema, alpha,
                                   static_cast<char *>(workspace), static_cast<hipStream_t>(hip_stream));
}

// ------------------------------------------------------------------------------------ debug validator
size_t dsv_idx_validate_workspace(const dsv_problem *p)
{
    if (check_problem(p, false) != DSV_OK) return 0;
    return 256;
}

dsv_status dsv_idx_validate(const dsv_problem *p, const int32_t *idx, int64_t *report, void *workspace,
                            size_t ws_bytes, void *hip_stream)
{
    dsv_status st = check_problem(p, false);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({idx})) return DSV_EINVAL;
    st = check_workspace(workspace, ws_bytes, 256);
    if (st != DSV_OK) return st;
    const std::vector<HeadTable> tabs = make_tables(*p);
    return launch_idx_validate(*p, tabs.data(), (int)tabs.size(), idx, static_cast<unsigned long long *>(workspace),
                               report, static_cast<hipStream_t>(hip_stream));
}

// ------------------------------------------------------------------------------------ parity exports
dsv_status dsv_lowrank_project(const dsv_problem *p, const void *Q, const void *K, const void *Wq, const void *Wk,
                               void *Qlr, void *Klr, void *hip_stream)
{
    dsv_status st = check_problem(p, true);
    if (st != DSV_OK) return st;
    if (!ok_ptrs({Q, K, Wq, Wk, Qlr, Klr})) return DSV_EINVAL;
    return launch_project(*p, p->L, Q, K, Wq, Wk, Qlr, Klr, static_cast<hipStream_t>(hip_stream));
}

dsv_status dsv_lowrank_scores_rows(const dsv_problem *p, const void *Qlr, const void *Klr, int32_t b, int32_t h,
                                   const int32_t *rows, int32_t n_rows, float *scores, void *hip_stream)
{
    dsv_status st = check_problem(p, true);
    if (st != DSV_OK) return st;
    if (!rows || !scores || n_rows < 1) return DSV_EINVAL;
    if (b < 0 || b >= p->B || h < 0 || h >= p->H) return DSV_EINVAL;
    if (!ok_ptrs({Qlr, Klr})) return DSV_EINVAL;
    return launch_scores_rows(*p, Qlr, Klr, b * p->H + h, rows, n_rows, scores, static_cast<hipStream_t>(hip_stream));
}

// ------------------------------------------------------------------------------------ measurement aid
dsv_status dsv_kernel_timing(int32_t enable)
{
    dsv::KernelTimer &t = dsv::g_kernel_timer;
    if (enable && !t.ev[0][0]) {
        for (int i = 0; i < DSV_KERNEL_COUNT; ++i)
            for (int e = 0; e < 2; ++e)
                if (hipEventCreate(&t.ev[i][e]) != hipSuccess) return DSV_EHIP;
    }
    for (int i = 0; i < DSV_KERNEL_COUNT; ++i) t.recorded[i] = false;
    t.on = enable != 0;
    return DSV_OK;
}

int32_t dsv_threshold_search(int32_t mode)
{
    if (mode < 0 || mode > 2) return -1;
    return dsv::set_threshold_search(mode);
}

int32_t dsv_threshold_sample_keys(int32_t L, int32_t k)
{
    const int mode = dsv::set_threshold_search(-1);
    return mode == 1 ? 0 : dsv::window_sample_keys(L, k, mode == 2);
}

dsv_status dsv_kernel_ms(int32_t span, float *ms)
{
    dsv::KernelTimer &t = dsv::g_kernel_timer;
    if (!ms || span < 0 || span >= DSV_KERNEL_COUNT || !t.recorded[span]) return DSV_EINVAL;
    if (hipEventSynchronize(t.ev[span][1]) != hipSuccess) return DSV_EHIP;
    if (hipEventElapsedTime(ms, t.ev[span][0], t.ev[span][1]) != hipSuccess) return DSV_EHIP;
    return DSV_OK;
}

}  // extern "C"
