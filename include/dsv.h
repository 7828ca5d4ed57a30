/*
 * dsv.h -- C ABI of libdsv: the two-stage dynamic sparse attention of DSV on one MI355X (gfx950).
 *
 * Stage 1 (dsv_lowrank_topk) estimates, for every (head, query), which k keys matter most, from
 * low-rank projections of Q and K; stage 2 (dsv_sparse_attn_fwd / dsv_sparse_attn_bwd) computes
 * exact softmax attention, and its gradients, over only those keys.
 *
 * Conventions that hold for every entry point
 *   - Tensor pointers are DEVICE pointers owned by the caller, contiguous, row-major, no strides:
 *       Q, K, V, O, dO, dQ, dK, dV : [B, H, L, d]   element type dsv_problem.dtype
 *       Wq, Wk                     : [H, d, r]      same element type (one predictor pair per head)
 *       lse                        : [B, H, L]      float
 *       idx                        : ragged int32; the block of (b, h) starts at element
 *                                    off[b*H+h] = sum over earlier (b', h') of L * k_per_head[h'],
 *                                    and holds [L, k_h] row-major (dsv_idx_offsets computes off).
 *     dsv_problem and the arrays it points to (k_per_head) are HOST memory, read during the call.
 *   - The library allocates and frees no device memory and keeps no state between calls (the
 *     optional measurement aid at the end of this header aside).  Scratch
 *     comes from the caller: ask dsv_*_workspace() for the size, pass a device buffer of at least
 *     that many bytes, aligned to 256 bytes.  Its contents are undefined afterwards.
 *   - Work is enqueued on the caller's HIP stream (hip_stream is a hipStream_t; NULL = the default
 *     stream) and the call returns once it is enqueued.  Outputs are fully overwritten.
 *   - Errors come back as a dsv_status; nothing is thrown or aborted across the boundary.  Argument
 *     errors (null pointer, k_h outside [1, L], unsupported d / r / dtype, workspace too small) are
 *     found on the host before anything is launched.
 *   - idx contract: every value in [0, L), values distinct within a row.  dsv_lowrank_topk writes
 *     rows in ascending key index.  The stage-2 calls accept rows in any order.  Rows that break
 *     the contract give undefined results; the stage-2 calls never check them (dsv_idx_validate does,
 *     on request).
 *   - Supported: d in {64, 128}; r in {16, 32, 64}; dtype F32 or BF16; 1 <= B*H <= 65535; L >= 1 with
 *     one head's [L, d] matrix below 4 GB (L < 2^24 for bf16, d = 128); anything else: DSV_EUNSUPPORTED
 *     (B*H out of range: DSV_EINVAL).
 *   - Inputs are assumed finite (no NaN / Inf).
 *
 * Paper: "DSV: Exploiting Dynamic Sparsity to Accelerate Large-Scale Video DiT Training".
 */
#ifndef DSV_H_
#define DSV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define DSV_API __attribute__((visibility("default")))
#else
#define DSV_API
#endif

typedef enum { DSV_F32 = 0, DSV_BF16 = 1 } dsv_dtype;

typedef enum {
    DSV_OK = 0,
    DSV_EINVAL = -1,        /* bad argument: null pointer, size out of range, k_h not in [1, L] */
    DSV_EUNSUPPORTED = -2,  /* d, r or dtype outside the supported set */
    DSV_EWORKSPACE = -3,    /* workspace pointer null / misaligned, or ws_bytes too small */
    DSV_EHIP = -4           /* a HIP runtime call or a kernel launch reported an error */
} dsv_status;

/* Problem descriptor shared by all calls (host memory). */
typedef struct dsv_problem {
    int32_t B;                  /* batch */
    int32_t H;                  /* heads held by this GPU */
    int32_t L;                  /* tokens (the paper's S): queries and keys alike */
    int32_t d;                  /* head dimension */
    int32_t r;                  /* predictor rank (the paper's d_lr); ignored by stage 2 */
    int32_t dtype;              /* dsv_dtype of Q, K, V, Wq, Wk, O, dO, dQ, dK, dV */
    const int32_t *k_per_head;  /* HOST array [H]: KV kept per query in head h, 1 <= k_h <= L
                                   (one sparsity level per head: Sec. "Limitations and Future Work") */
    float scale;                /* softmax scale applied to q.k; the paper uses 1/sqrt(d_k) */
    uint32_t flags;             /* DSV_FLAG_* bits, 0 for none */
} dsv_problem;

/* The caller promises that every idx row, and every idx_t list, is in ascending order -- which is
 * how dsv_lowrank_topk / dsv_lowrank_topk_t write them.  Stage 2 then runs its L2-blocked kernels
 * (the key axis cut into cache-sized ranges, one contiguous segment of each row per range), which
 * need more workspace and are several times faster on long sequences.  Without the flag stage 2
 * makes no assumption on the order.  Setting it for unsorted indices gives wrong results. */
#define DSV_FLAG_SORTED_INDEX 1u

DSV_API const char *dsv_version(void);
DSV_API const char *dsv_status_string(dsv_status s);

/* Writes off[0 .. B*H] (HOST int64 array of B*H+1 entries): element offsets of each (b, h) block
 * of idx; off[B*H] is the total element count.  Returns DSV_EINVAL on a bad descriptor. */
DSV_API dsv_status dsv_idx_offsets(const dsv_problem *p, int64_t *off);

/* ---- Stage 1: critical-KV estimation ------------------------------------------------------
 * Sec. "Low-Rank based Sparsity Prediction" (Q_lr = Q Wq, K_lr = K Wk with inner dimension r)
 * and Sec. "Critical KV Estimation with Kernel Fusion" (top-k of every row of Q_lr K_lr^T,
 * fused with the product so that the [H, L, L] score tensor is never stored); the two-pass
 * form -- find each query's threshold, then select against it -- is the one Appendix
 * "Implementation details" gives for large k.
 *
 * For every (b, h, i): idx row = the k_h keys j with the largest score
 *     s_ij = sum_t Q_lr[i, t] * K_lr[j, t],
 * Q_lr, K_lr rounded to `dtype`, s accumulated in fp32 on the matrix cores; equal scores go to
 * the lower key index; the row is written in ascending key index; exactly k_h entries.
 * Needs workspace (projections and per-query selection state). */
DSV_API size_t dsv_lowrank_topk_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_lowrank_topk(const dsv_problem *p, const void *Q, const void *K,
                            const void *Wq, const void *Wk, int32_t *idx,
                            void *workspace, size_t ws_bytes, void *hip_stream);

/* Same selection, and in addition its transpose: idx_t / col_ptr in the layout dsv_idx_transpose
 * documents below, with every key's query list in ASCENDING query order.  The key-major lists are
 * emitted by re-evaluating the selection predicate key tile by key tile (two more sweeps over the
 * scores), which is much cheaper than sorting the emitted pairs by key, and is what lets the
 * backward's dkdv step run without building the lists itself. */
DSV_API size_t dsv_lowrank_topk_t_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_lowrank_topk_t(const dsv_problem *p, const void *Q, const void *K,
                                      const void *Wq, const void *Wk, int32_t *idx, int32_t *idx_t,
                                      int64_t *col_ptr, void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Stage 2 forward: attention over the selected KV only -----------------------------------
 * Sec. "Sparse Attention with Query Grouping" (per-query form, no grouping) with the softmax
 * attention of Sec. "Various Self-Attention Paradigms":
 *     s_j = scale * q_i . k_j  for j in idx row (b, h, i);   p = softmax over those j only;
 *     O_i = sum_j p_j v_j;     lse_i = log sum_j exp(s_j).
 * O is written in `dtype`, lse in float.  Workspace: none without DSV_FLAG_SORTED_INDEX (the query
 * returns 0 and a null workspace is accepted); with it, the segment pointers and the per-range
 * partial results. */
DSV_API size_t dsv_sparse_attn_fwd_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_sparse_attn_fwd(const dsv_problem *p, const void *Q, const void *K, const void *V,
                               const int32_t *idx, void *O, float *lse,
                               void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Stage 2 backward ------------------------------------------------------------------------
 * Gradient of the forward above with the selection held constant (the predictor is trained
 * outside the main graph: Sec. "Low-Rank based Sparsity Prediction"), given O and lse from
 * dsv_sparse_attn_fwd and the upstream gradient dO:
 *     Delta_i = dO_i . O_i;  p_ij = exp(s_ij - lse_i);  dS_ij = p_ij (dO_i . v_j - Delta_i);
 *     dQ_i = scale sum_j dS_ij k_j;
 *     dK_j = scale sum_{i: j in row i} dS_ij q_i;   dV_j = sum_{i: j in row i} p_ij dO_i.
 * Keys no query selected get zeros.  dQ, dK, dV are written in `dtype` (accumulated in fp32).
 * Delta is formed from the per-pair terms in fp32 rather than from the storage-rounded O, whose
 * rounding alone would cost more than the output tolerance; O only serves as a centring value
 * (dO . O is within rounding of Delta) that keeps the accumulated weights small.  The workspace holds Delta, the transposed index
 * (as large as idx), its column pointers and the counters of dsv_idx_transpose.  The transposed index built here has
 * ascending lists whatever the order inside the rows of idx is, so the dkdv step always runs its L2-blocked kernel
 * and the results are identical, bit for bit, to dsv_sparse_attn_bwd_t on dsv_idx_transpose's output and from run to
 * run.  The transposition is a scatter of 4-byte entries and costs more than either sweep on long sequences
 * (L = 131072, k = 8192, 6 heads: 640 ms of 910); callers that run stage 1 here should take its transposed index
 * (dsv_lowrank_topk_t) and call dsv_sparse_attn_bwd_t. */
DSV_API size_t dsv_sparse_attn_bwd_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_sparse_attn_bwd(const dsv_problem *p, const void *Q, const void *K, const void *V,
                               const int32_t *idx, const void *O, const float *lse, const void *dO,
                               void *dQ, void *dK, void *dV,
                               void *workspace, size_t ws_bytes, void *hip_stream);

/* Whole backward with the transposed index supplied by the caller (from dsv_lowrank_topk_t, or
 * from an earlier dsv_idx_transpose): dq step then dkdv step; nothing is built here, so with
 * DSV_FLAG_SORTED_INDEX both steps run L2-blocked.  Same outputs as dsv_sparse_attn_bwd. */
DSV_API size_t dsv_sparse_attn_bwd_t_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_sparse_attn_bwd_t(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                         const int32_t *idx, const int32_t *idx_t, const int64_t *col_ptr,
                                         const void *O, const float *lse, const void *dO,
                                         void *dQ, void *dK, void *dV,
                                         void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- The steps of the backward, callable one by one ----------------------------------------------
 * dsv_sparse_attn_bwd runs dq, transpose, dkdv in this order (dsv_sparse_attn_bwd_t: dq, dkdv).
 * They are exported so that a caller can keep the transposed index across calls that share idx,
 * and so that each step can be timed on its own.
 *
 * dsv_sparse_attn_bwd_dq: query-major sweep.  Writes dQ [B, H, L, d] (`dtype`) and
 *   delta [B, H, L] (float) = Delta_i = sum_j p_ij (dO_i . v_j), which equals dO_i . O_i.
 *
 * dsv_idx_transpose: for every (b, h) and key j, the list of queries i whose idx row holds j.
 *   idx_t: int32, same ragged layout and size as idx (per head, the lists of key 0, 1, ... back to
 *   back); col_ptr: int64 [B*H, L+1], list of key j of head bh = idx_t[off[bh] + col_ptr[bh][j] ..
 *   off[bh] + col_ptr[bh][j+1]).  A stable counting sort: every list is in ascending query order whatever the
 *   order inside the rows of idx is, and the output is the same from run to run; for rows as stage 1 writes them
 *   it equals dsv_lowrank_topk_t's idx_t.  Workspace: int32 counters per (b, h, key) and per (b, h, chunk of
 *   query rows, key), at most 257 per (b, h, key).
 *
 * dsv_sparse_attn_bwd_dkdv: key-major sweep over idx_t.  Writes dK, dV [B, H, L, d] (`dtype`);
 *   keys with an empty list get zeros.
 *
 * Workspace of dq and dkdv: none without DSV_FLAG_SORTED_INDEX (query returns 0, null accepted);
 * with it, segment pointers and per-range partial sums. */
DSV_API size_t dsv_sparse_attn_bwd_dq_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_sparse_attn_bwd_dq(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                          const int32_t *idx, const void *O, const float *lse, const void *dO,
                                          void *dQ, float *delta,
                                          void *workspace, size_t ws_bytes, void *hip_stream);
DSV_API size_t dsv_idx_transpose_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_idx_transpose(const dsv_problem *p, const int32_t *idx, int32_t *idx_t, int64_t *col_ptr,
                                     void *workspace, size_t ws_bytes, void *hip_stream);
DSV_API size_t dsv_sparse_attn_bwd_dkdv_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_sparse_attn_bwd_dkdv(const dsv_problem *p, const void *Q, const void *K, const void *V,
                                            const int32_t *idx_t, const int64_t *col_ptr, const float *lse,
                                            const float *delta, const void *dO, void *dK, void *dV,
                                            void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Query grouping ----------------------------------------------------------------------------
 * Sec. "Sparse Attention with Query Grouping" (with Observation 5: neighbouring tokens of the 3D latent
 * grid attend to similar keys): the tokens lie on a grid of F x Hh x Ww (token index
 * (f * Hh + h) * Ww + w: frames first, then height, then width); the grid is tiled by cubes of
 * gf x gh x gw voxels; the G = gf*gh*gw queries of a cube share ONE index row, chosen by the cube's
 * centre query alone (the voxel at offset (gf/2, gh/2, gw/2) of the cube).  Groups are numbered like
 * tokens (cube coordinates, frames first), members likewise inside their cube.
 * Requires F*Hh*Ww == L and gf | F, gh | Hh, gw | Ww; anything else: DSV_EINVAL.
 *
 * Grouped index layout: idx_g is ragged int32 like idx, the block of (b, h) holding [L/G, k_h]
 * (one row per group, ascending keys) at element off[b*H+h] / G of dsv_idx_offsets.  idx_t_g / col_ptr:
 * per key the ASCENDING list of GROUPS whose row holds it (col_ptr [B*H, L+1] as for idx_t).
 *
 * dsv_lowrank_topk_grouped: stage 1 on the centre queries only (1/G of the scoring and selection
 *   work).  idx_t_g and col_ptr may both be NULL (no key-major lists).
 * dsv_sparse_attn_fwd_grouped: every member of a group attends over the group's row; same O, lse as
 *   dsv_sparse_attn_fwd on the index with that row repeated for every member.  Each selected K / V
 *   row is gathered once per group and used by all members (both products of a tile on the matrix cores)
 *   for bf16, d = 128, G <= 32 (up to 8 members: one wave per group; up to 16 / 32: one block of two / four waves per
 *   group, sharing the gathered rows).  Every other dtype, head dimension or cube (G <= 64; larger: DSV_EUNSUPPORTED)
 *   gives the same results through the per-query kernels on queries reordered group by group, with the
 *   index expanded to one row per query in the workspace -- the contract without the saving.  With
 *   DSV_FLAG_SORTED_INDEX (rows ascending, as stage 1 writes them) the L2-blocked form runs and needs
 *   workspace (segment pointers, per-range partials); without the flag the group kernels need none (the
 *   query returns 0).
 * dsv_sparse_attn_bwd_grouped: gradients of the above (selection held constant).  dQ group by group with
 *   the forward's tiling (K and V rows gathered once per group); dK and dV with the per-query key-major
 *   sweep on queries reordered group by group: the workspace holds the reordered Q, dO, lse, Delta besides
 *   the steps' scratch, and -- unless the group kernels run with the flag set, where the sweep reads the lists
 *   of groups as they are -- the per-query form of the key-major index (L*k int32 per head).  Needs idx_t_g
 *   and col_ptr.  The flag selects the L2-blocked dQ step as in the forward.  Cases outside bf16, d = 128,
 *   G <= 32: dQ by the per-query kernel as described for the forward. */
typedef struct dsv_grouping {
    int32_t F, Hh, Ww;   /* token grid: frames, height, width */
    int32_t gf, gh, gw;  /* cube (group) size along each axis */
} dsv_grouping;

/* Offline profiling of the group size (same section: the largest cube whose queries share a required ratio, e.g.
 * 80 %, of their critical keys).  Given the PER-QUERY index idx (dsv_lowrank_topk; rows in any order) and a cube,
 *     overlap[b*H+h] = (1 / (L k_h)) sum_i | row(i) intersect row(centre query of i's group) |,
 * the mean share of a query's own selection that the shared row would keep (a centre query counts in full).
 * overlap: DEVICE float [B*H].  Workspace: one 64-bit counter per (b, h).  L <= 524288 (the centre's row is held as a
 * bitmap in LDS); larger: DSV_EUNSUPPORTED.
 *
 * dsv_choose_grouping: evaluates n candidate cubes (cubes: HOST int32 [n][3] = gf, gh, gw; candidates that do not
 * tile the F x Hh x Ww grid are skipped) and writes to *chosen (HOST) the index of the candidate with the most
 * members whose overlap is at least min_overlap in EVERY (b, h) -- the first such on ties -- or -1 if none is.
 * overlaps (HOST float [n][B*H], may be NULL) receives every candidate's figures (-1 for skipped ones).  Waits for
 * the stream.  Workspace: dsv_group_overlap's plus one float per (b, h). */
DSV_API size_t dsv_group_overlap_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_group_overlap(const dsv_problem *p, const dsv_grouping *g, const int32_t *idx, float *overlap,
                                     void *workspace, size_t ws_bytes, void *hip_stream);
DSV_API size_t dsv_choose_grouping_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_choose_grouping(const dsv_problem *p, int32_t F, int32_t Hh, int32_t Ww, const int32_t *cubes,
                                       int32_t n, const int32_t *idx, float min_overlap, int32_t *chosen,
                                       float *overlaps, void *workspace, size_t ws_bytes, void *hip_stream);

DSV_API size_t dsv_lowrank_topk_grouped_workspace(const dsv_problem *p, const dsv_grouping *g);
DSV_API dsv_status dsv_lowrank_topk_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                            const void *Wq, const void *Wk, int32_t *idx_g, int32_t *idx_t_g,
                                            int64_t *col_ptr, void *workspace, size_t ws_bytes, void *hip_stream);
DSV_API size_t dsv_sparse_attn_fwd_grouped_workspace(const dsv_problem *p, const dsv_grouping *g);
DSV_API dsv_status dsv_sparse_attn_fwd_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                               const void *V, const int32_t *idx_g, void *O, float *lse,
                                               void *workspace, size_t ws_bytes, void *hip_stream);
DSV_API size_t dsv_sparse_attn_bwd_grouped_workspace(const dsv_problem *p, const dsv_grouping *g);
DSV_API dsv_status dsv_sparse_attn_bwd_grouped(const dsv_problem *p, const dsv_grouping *g, const void *Q, const void *K,
                                               const void *V, const int32_t *idx_g, const int32_t *idx_t_g,
                                               const int64_t *col_ptr, const void *O, const float *lse, const void *dO,
                                               void *dQ, void *dK, void *dV, void *workspace, size_t ws_bytes,
                                               void *hip_stream);

/* ---- Predictor side: approximation loss and its gradients ---------------------------------------
 * Sec. "Low-Rank based Sparsity Prediction": the predictor (Wq, Wk) of a block is trained so that
 * Q_lr K_lr^T tracks Q K^T, with the loss 0.95 * CosLoss + 0.05 * NormLoss evaluated on a random sample of
 * query rows, in the forward pass, without storing Q K^T.  Per (b, h), with A = Q_s K^T and
 * Ahat = (Q_s Wq)(K Wk)^T over the n_rows sampled queries and all L keys:
 *     CosLoss  = mean_i ( 1 - <ahat_i, a_i> / (|ahat_i| |a_i|) )      (cosine of a query's score rows)
 *     NormLoss = mean_ij (ahat_ij - a_ij)^2
 * (no softmax scale; projections in full precision -- rounding belongs to the selection path).
 * rows: DEVICE int32 [n_rows], the sampled query rows (each in [0, L); the same rows for every head).
 * loss: DEVICE float [B*H, 3] = {0.95 Cos + 0.05 Norm, CosLoss, NormLoss}; dWq, dWk: DEVICE float
 * [B*H, d, r], the gradients of (b, h)'s loss (a caller with B > 1 sums them over b).
 * No row of A or Ahat is formed: everything is a quadratic form in the Gram matrix K^T K, the one pass
 * over the keys. */
DSV_API size_t dsv_predictor_loss_workspace(const dsv_problem *p, int32_t n_rows);
DSV_API dsv_status dsv_predictor_loss(const dsv_problem *p, const void *Q, const void *K, const void *Wq,
                                      const void *Wk, const int32_t *rows, int32_t n_rows, float *loss, float *dWq,
                                      float *dWk, void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Predictor side: sparsity profiler --------------------------------------------------------------
 * Sec. "Sparsity Profiling": the sparsity of every head is measured on a sample of query rows from the softmax
 * of the true scores (scale * Q K^T over all L keys) and kept as an exponential moving average.  Definition
 * (Sec. "Exploiting Dynamic Sparsity"): a query's critical KV are its highest-probability keys that together
 * hold `mass` of its softmax (the paper: 0.9); the head's sparsity is the mean fraction of NON-critical keys.
 * rows: DEVICE int32 [n_rows] (each in [0, L); the same rows for every head); 0 < mass < 1.
 * counts: DEVICE int32 [B*H, n_rows], the number of critical keys of every sampled query;
 * sparsity: DEVICE float [B*H] = mean_i (1 - counts_i / L);
 * ema: DEVICE float [B*H] or NULL: updated in place, ema = alpha * sparsity + (1 - alpha) * ema.
 * Scores are recomputed in each of five sweeps on the matrix cores, never stored.  A count can differ by
 * one key between runs (probability mass is summed with LDS float atomics). */
DSV_API size_t dsv_profile_sparsity_workspace(const dsv_problem *p, int32_t n_rows);
DSV_API dsv_status dsv_profile_sparsity(const dsv_problem *p, const void *Q, const void *K, const int32_t *rows,
                                        int32_t n_rows, float mass, int32_t *counts, float *sparsity, float *ema,
                                        float alpha, void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Optional debug check of an index tensor ---------------------------------------------------
 * Checks every row of idx against the idx contract above: values in [0, L), distinct within a row,
 * and -- when dsv_problem.flags has DSV_FLAG_SORTED_INDEX -- strictly ascending (which is what the
 * L2-blocked stage-2 kernels rely on).  Unlike every other call this one WAITS for the stream: it
 * returns DSV_OK when all rows are valid and DSV_EINVAL when any row is not.
 * report: HOST int64 [3], may be NULL: {number of offending rows, b*H+h of the first one, its row}
 * (first = smallest (b*H+h, row); -1, -1 when there is none).
 * Without the flag the duplicate check keeps a bitmap of L bits in LDS: L <= 524288, else
 * DSV_EUNSUPPORTED.  Workspace: 256 bytes (counters). */
DSV_API size_t dsv_idx_validate_workspace(const dsv_problem *p);
DSV_API dsv_status dsv_idx_validate(const dsv_problem *p, const int32_t *idx, int64_t *report,
                                    void *workspace, size_t ws_bytes, void *hip_stream);

/* ---- Stage 1 for callers that cannot allocate -------------------------------------------------
 * For callers that can neither allocate device memory nor bring a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same operation, same result as
 * dsv_lowrank_topk, but the scratch (projections and per-query selection state) lives in a
 * fixed array inside the library's device image instead of a caller's workspace: the call
 * allocates nothing and frees nothing.
 * Limit: dsv_lowrank_topk_workspace(p) <= dsv_lowrank_topk_noalloc_max_bytes() (32 MiB: e.g.
 * bf16, r = 16, B*H*L up to about 450 000 tokens); larger problems: DSV_EWORKSPACE, nothing launched.
 * Every GPU the library runs on holds its own copy of the array until the process ends.  All calls
 * on one GPU share it: calls that overlap on one GPU (two streams, two threads) race; run them
 * one after another.  The array keeps the previous call's contents; the call itself (re)writes
 * everything it reads. */
DSV_API size_t dsv_lowrank_topk_noalloc_max_bytes(void);
DSV_API dsv_status dsv_lowrank_topk_noalloc(const dsv_problem *p, const void *Q, const void *K,
                                            const void *Wq, const void *Wk, int32_t *idx, void *hip_stream);

/* ---- Stage-1 internals exported for parity checks ---------------------------------------------
 * dsv_lowrank_project: only the projection step of stage 1 (Sec. "Low-Rank based Sparsity
 * Prediction").  Qlr, Klr: [B, H, L, r] in `dtype`, no padding.  No workspace.
 *
 * dsv_lowrank_scores_rows: the fp32 scores exactly as the selection kernels compute them (same
 * matrix-core instruction sequence), for n_rows chosen queries of one (b, h).  Qlr, Klr as written
 * by dsv_lowrank_project; rows: DEVICE int32 [n_rows], each in [0, L); scores: DEVICE float
 * [n_rows, L].  No workspace. */
DSV_API dsv_status dsv_lowrank_project(const dsv_problem *p, const void *Q, const void *K,
                               const void *Wq, const void *Wk, void *Qlr, void *Klr,
                               void *hip_stream);
DSV_API dsv_status dsv_lowrank_scores_rows(const dsv_problem *p, const void *Qlr, const void *Klr,
                                   int32_t b, int32_t h, const int32_t *rows, int32_t n_rows,
                                   float *scores, void *hip_stream);

/* ---- measurement aid -------------------------------------------------------------------------
 * Not an operation of the method: lets a benchmark time single kernels inside the calls above with
 * HIP events on the stream they are launched on.
 * dsv_kernel_timing(1): from now on every call records a pair of events around each kernel span
 * listed below (created on the current device at the first enable); (0) switches that off.
 * Process-wide and not thread-safe; off by default; with it on, calls must not be captured into a
 * HIP graph.
 * dsv_kernel_ms: waits for the span's stop event of the most recent call that ran it and writes the
 * elapsed milliseconds to *ms (HOST).  DSV_EINVAL if the span has not run since timing was enabled.
 * When a call launches a span's kernel once per group of up to 64 heads, the span covers all of
 * those launches. */
typedef enum {
  DSV_KERNEL_FWD_SWEEP = 0,   /* sparse forward gather sweep */
  DSV_KERNEL_DQ_SWEEP = 1,    /* backward, query-major sweep */
  DSV_KERNEL_DKDV_SWEEP = 2,  /* backward, key-major sweep */
  DSV_KERNEL_THRESHOLD = 3,   /* stage 1: all kernels of the threshold search together */
  DSV_KERNEL_EMIT = 4,        /* stage 1: query-major emission */
  DSV_KERNEL_EMIT_T_COUNT = 5,/* stage 1: key-major counting pass */
  DSV_KERNEL_EMIT_T_WRITE = 6,/* stage 1: key-major emission */
  DSV_KERNEL_COUNT = 7
} dsv_kernel_span;
DSV_API dsv_status dsv_kernel_timing(int32_t enable);
DSV_API dsv_status dsv_kernel_ms(int32_t span, float *ms);

/* How stage 1 finds every query's threshold score (the k-th largest; paper Sec. "Critical KV Estimation with
 * Kernel Fusion").  Both methods are exact and give identical results; the choice only affects speed.
 *   0  automatic (default): the windowed search -- a key sample brackets the threshold, then two sweeps over
 *      the keys -- for heads with L >= 16384 and k <= L/4 whose sample (2048 to 16384 keys, at most L/8) holds
 *      enough keys on both sides of the threshold; else the radix search (four sweeps, 8 bits each);
 *   1  always the radix search;
 *   2  the windowed search for every head it can serve at all (L >= 4096, sample up to L/2 keys).
 * Query tiles the windowed search cannot settle (threshold outside the bracket, massive ties) go through the
 * radix search afterwards, inside the same call.  Process-wide; for tests and measurements.  Returns the
 * previous mode; a mode outside 0..2 changes nothing and returns -1. */
DSV_API int32_t dsv_threshold_search(int32_t mode);
/* Which search a head that keeps k of L keys gets under the current mode: the number of keys the windowed
 * search samples for it (a multiple of 32), or 0 when the head takes the radix search.  Host arithmetic only. */
DSV_API int32_t dsv_threshold_sample_keys(int32_t L, int32_t k);

/* Pure-gather probe: the practical ceiling of the vector memory path (L2 -> vector L1 -> registers) for the
 * stage-2 access pattern, against which the sweeps' achieved gather rate is reported.  K, V: DEVICE bf16
 * [n_ranges * range_rows, 128]; idx: DEVICE int32 [n_ranges, idx_rows, k], every row an ascending list of row
 * numbers inside one range (0 .. range_rows - 1); nq query rows per range use index row (q mod idx_rows), so
 * idx_rows = nq streams the index from memory as the real sweeps do and a small idx_rows keeps it cached.
 * Every query gathers, per index entry, one K row and one V row of the range (2 x 256 bytes) with the forward
 * sweep's lane layout, index staging and XCD-aware block order, and does no arithmetic on them.
 * out: DEVICE uint32 [n_ranges, nq].  Runs the kernel once untimed, then `reps` times, and writes the mean
 * milliseconds per launch to *ms (HOST); waits for the stream.  k must be a multiple of 4.
 * Gathered bytes per launch = n_ranges * nq * k * 512. */
DSV_API dsv_status dsv_measure_gather_ceiling(int32_t n_ranges, int32_t range_rows, int32_t nq, int32_t k,
                                              int32_t idx_rows, const void *K, const void *V, const int32_t *idx,
                                              void *out, int32_t reps, float *ms, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* DSV_H_ */
