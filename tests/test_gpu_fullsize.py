"""Parity at the benchmark configurations' full sizes, in the launch configuration bench.py times:
sorted-index flag set, stage 1 emitting the transposed index, backward through dsv_sparse_attn_bwd_t.
Configs 1-4 of the benchmark list (config 0 is small enough to be checked in full elsewhere); config 2
is the one bench.py reports.

The oracle cannot do whole problems of this size (1e11 and more scores), so it computes sampled outputs
one by one:
  * stage 1 on the real top-k: sampled index rows against the oracle's selection applied to the
    device's own fp32 score bits (bit-exact) and against the pure fp64 oracle; the whole index identical
    under both threshold searches; properties that hold
    at any size for everything else (rows ascending and in range, exactly k per row, idx_t is the
    exact transpose of idx for sampled keys, list lengths = per-key counts);
  * stage 2 on that real selection (what the benchmark runs): forward and backward_t on the device's
    idx / idx_t; O, lse, dQ of the sampled rows -- whose index rows were just shown bit-exact -- against
    the oracle, and dK, dV of sampled keys, among them the key with the longest list and the one with
    the shortest, each list first checked against the column of idx by a plain device comparison;
  * stage 2 on a synthetic index tensor whose rows AND columns have a closed form (arithmetic
    progressions modulo L, from the workload generator): the same outputs with an index no device
    code produced (uniform list lengths: the complement of the skewed real selection);
  * the query-grouped variant (configs 1 and 2, 2 x 2 x 2 cubes) the same way on its own real selection.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import assert_close, assert_t3_valid, score_error_bound

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")

CONFIGS = (1, 2, 3, 4)


def _host_heads(cfg):
    return (0, cfg.H - 1)      # heads whose inputs are also kept on the host for the oracle


def _row_chunks(L, k, elems=1 << 28):
    """Row ranges of an [L, k] tensor with at most `elems` elements each (torch temporaries stay small)."""
    step = max(1, elems // k)
    return [(lo, min(lo + step, L)) for lo in range(0, L, step)]


@pytest.fixture(scope="module", params=CONFIGS, ids=lambda c: f"config{c}")
def data(request, progress):
    cfg = wl.get_config(request.param)
    ks = [int(x) for x in wl.k_per_head(cfg)]
    td = torch.bfloat16
    dev = "cuda:0"
    g = {n: torch.empty((1, cfg.H, cfg.L, cfg.d), dtype=td, device=dev) for n in ("Q", "K", "V", "dO")}
    Wq = torch.empty((cfg.H, cfg.d, cfg.r), dtype=td, device=dev)
    Wk = torch.empty((cfg.H, cfg.d, cfg.r), dtype=td, device=dev)
    host = {}
    for h in range(cfg.H):
        t = wl.head_tensors(cfg, h)
        for n in g:
            g[n][0, h].copy_(torch.from_numpy(t[n]).to(td))
        wq, wk = wl.predictor_weights(cfg, h)
        Wq[h].copy_(torch.from_numpy(wq).to(td))
        Wk[h].copy_(torch.from_numpy(wk).to(td))
        if h in _host_heads(cfg):
            host[h] = dict(t, Wq=wq, Wk=wk)
        if cfg.L >= 1 << 18:
            progress(f"config {cfg.index}: head {h} generated")
    progress(f"config {cfg.index}: inputs generated")
    yield cfg, ks, g, Wq, Wk, host
    del g, Wq, Wk
    torch.cuda.empty_cache()


N_ROWS = 64          # sampled query rows per checked head (plus the first and the last row)
N_KEYS = 8           # sampled keys per config for dK / dV (longest list, shortest list, random ones)
MAX_LIST = 100_000   # the oracle walks every selecting query's whole row: longest list checked is capped here


def _column_of(idx_rows, j, L, k):
    """Queries whose index row holds key j, by a plain comparison on the device (no library call)."""
    hit = torch.cat([(idx_rows[lo:hi] == j).any(dim=1) for lo, hi in _row_chunks(L, k)])
    return torch.nonzero(hit).reshape(-1)


def test_real_selection_full_size(data, progress):
    """Stage 1 at full size, then stage 2 forward and backward on the index stage 1 wrote (the
    benchmark's path: lowrank_topk_t -> sparse_attn_fwd -> sparse_attn_bwd_t on the device's idx / idx_t)."""
    cfg, ks, g, Wq, Wk, host = data
    L = cfg.L
    off = wl.idx_offsets(1, cfg.H, L, ks)
    p = dsv.Problem(1, cfg.H, L, cfg.d, cfg.r, cfg.dtype, ks, cfg.scale, sorted_index=True)
    idx_flat, idx_t_flat, col = dsv.lowrank_topk_t(p, g["Q"], g["K"], Wq, Wk)
    Qlr, Klr = dsv.lowrank_project(p, g["Q"], g["K"], Wq, Wk)
    torch.cuda.synchronize()
    progress(f"config {cfg.index}: stage 1 done")
    # the two threshold searches are both exact: every row of the index identical whichever one ran
    # (automatic choice above: the windowed search for the heads it fits; here the radix search for all)
    try:
        dsv.threshold_search(1)
        idx_radix = dsv.lowrank_topk(p, g["Q"], g["K"], Wq, Wk)
        torch.cuda.synchronize()
    finally:
        dsv.threshold_search(0)
    for lo in range(0, idx_flat.numel(), 1 << 30):
        assert torch.equal(idx_flat[lo:lo + (1 << 30)], idx_radix[lo:lo + (1 << 30)]), "windowed and radix search differ"
    del idx_radix
    torch.cuda.empty_cache()
    progress(f"config {cfg.index}: windowed = radix on all {idx_flat.numel()} index entries")

    def rows_of(h):
        return idx_flat[off[h]:off[h + 1]].view(L, ks[h])

    # any-size properties, all heads
    for h in range(cfg.H):
        idx = rows_of(h)
        for lo, hi in _row_chunks(L, ks[h]):
            part = idx[lo:hi]
            assert int(part.min()) >= 0 and int(part.max()) < L
            if ks[h] > 1:
                assert bool((part[:, 1:] > part[:, :-1]).all()), f"head {h}: rows not strictly ascending"
        assert int(col[h, 0]) == 0 and int(col[h, -1]) == L * ks[h]
        assert bool((col[h, 1:] >= col[h, :-1]).all())
    # list lengths = per-key counts, one head
    h = _host_heads(cfg)[1]
    counts = torch.zeros(L, dtype=torch.int64, device=idx_flat.device)
    for lo, hi in _row_chunks(L, ks[h]):
        counts += torch.bincount(rows_of(h)[lo:hi].reshape(-1), minlength=L)
    assert torch.equal(counts, col[h, 1:] - col[h, :-1])
    del counts
    rng = np.random.default_rng(0)
    sampled = {}
    for h in _host_heads(cfg):
        idx, k = rows_of(h), ks[h]
        idx_t = idx_t_flat[off[h]:off[h + 1]]
        # exact transpose for sampled keys
        for j in rng.integers(0, L, size=3).tolist() + [0, L - 1]:
            want = _column_of(idx, j, L, k).to(torch.int32)
            got = idx_t[int(col[h, j]):int(col[h, j + 1])]
            assert torch.equal(want, got), f"head {h} key {j}: idx_t list is not the column of idx"
        # sampled rows against the oracle
        rows = np.unique(np.concatenate([rng.integers(0, L, size=N_ROWS), [0, L - 1]])).astype(np.int32)
        S_gpu = dsv.lowrank_scores_rows(p, Qlr, Klr, 0, h, torch.from_numpy(rows).cuda())
        torch.cuda.synchronize()
        got = idx[torch.from_numpy(rows.astype(np.int64)).cuda()].cpu().numpy()
        # T2: the oracle's selection on the device's own fp32 score bits -> bit-exact
        t2 = oracle.topk_from_scores(S_gpu.cpu().numpy().astype(np.float64), k)
        assert np.array_equal(t2, got), f"head {h}: selection differs from the oracle's on the same score bits"
        # T3: against the pure fp64 oracle, differences only inside the rounding band of its threshold
        # (gpu_util.assert_t3_valid: |S_or[j] - tau_or| <= max_j' e[j'] + e[j])
        t3, _, _, S_or = oracle.lowrank_topk(host[h]["Q"][rows], host[h]["K"], host[h]["Wq"], host[h]["Wk"], k, cfg.dtype,
                                             return_intermediates=True)
        Qd = Qlr[0, h][torch.from_numpy(rows.astype(np.int64)).cuda()].float().cpu().numpy()
        Kd = Klr[0, h].float().cpu().numpy()
        S_dev_exact = oracle.scores(Qd, Kd)
        e = score_error_bound(Qd, Kd, S_dev_exact, S_or, cfg.r)
        assert np.all(np.abs(S_gpu.cpu().numpy() - S_dev_exact) <= e)
        same = sum(assert_t3_valid(f"config {cfg.index} head {h} row {rows[a]}", got[a], t3[a], S_or[a], e[a], k)
                   for a in range(len(rows)))
        del S_or, S_dev_exact, e, S_gpu
        progress(f"config {cfg.index} head {h}: {same}/{len(rows)} sampled rows identical to the pure fp64 oracle")
        sampled[h] = (rows.astype(np.int64), got)
    del Qlr, Klr
    torch.cuda.empty_cache()

    # ---- stage 2 on the device's own selection (rows just shown bit-exact on the device's score bits) ----
    O, lse = dsv.sparse_attn_fwd(p, g["Q"], g["K"], g["V"], idx_flat)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    dQ, dK, dV = dsv.sparse_attn_bwd_t(p, g["Q"], g["K"], g["V"], idx_flat, idx_t_flat, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    progress(f"config {cfg.index}: stage 2 on the real selection done")
    for h in _host_heads(cfg):
        t = host[h]
        rows, idx_rows = sampled[h]
        O_ref, lse_ref = oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], idx_rows, cfg.scale)
        dQ_ref = oracle.sparse_bwd_dq_rows(t["Q"][rows], t["K"], t["V"], idx_rows, t["dO"][rows], cfg.scale)
        sel = torch.from_numpy(rows).cuda()
        assert_close(f"O[h={h}]", O[0, h][sel], O_ref, cfg.dtype)
        assert_close(f"lse[h={h}]", lse[0, h][sel], lse_ref, "f32")
        assert_close(f"dQ[h={h}]", dQ[0, h][sel], dQ_ref, cfg.dtype)
    # dK, dV of sampled keys: every selecting query is needed -- the key's list, checked against the column of idx
    h = _host_heads(cfg)[0]
    t, k, idx = host[h], ks[h], rows_of(h)
    lens = (col[h, 1:] - col[h, :-1]).cpu().numpy()
    capped = np.where(lens <= MAX_LIST, lens, -1)
    keys = [int(capped.argmax()), int(lens.argmin())] + rng.integers(0, L, size=N_KEYS - 2).tolist()
    progress(f"config {cfg.index} head {h}: list lengths min {lens.min()} mean {lens.mean():.0f} max {lens.max()}")
    for j in keys:
        qs_dev = _column_of(idx, j, L, k)
        mine = idx_t_flat[off[h] + int(col[h, j]):off[h] + int(col[h, j + 1])]
        assert torch.equal(qs_dev.to(torch.int32), mine), f"key {j}: idx_t list is not the column of idx"
        qs = qs_dev.cpu().numpy()
        # the oracle's per-key routine, a chunk of the selecting queries at a time (its terms add over queries;
        # the chunks keep the fetched index rows small and the run talking)
        dKj, dVj = np.zeros(cfg.d), np.zeros(cfg.d)
        step = max(1, (1 << 27) // k)
        for lo in range(0, len(qs), step):
            part = qs[lo:lo + step]
            idx_sel = idx[qs_dev[lo:lo + step]].cpu().numpy()
            a, b = oracle.sparse_bwd_dkdv_key(j, t["Q"][part], t["dO"][part], idx_sel, t["K"], t["V"], cfg.scale)
            dKj += a
            dVj += b
            if len(qs) > step:
                progress(f"config {cfg.index} key {j}: {min(lo + step, len(qs))}/{len(qs)} selecting queries")
        if len(qs) == 0:
            assert float(dK[0, h, j].abs().max()) == 0.0 and float(dV[0, h, j].abs().max()) == 0.0
        assert_close(f"dK[h={h}, j={j}]", dK[0, h, j], dKj, cfg.dtype)
        assert_close(f"dV[h={h}, j={j}]", dV[0, h, j], dVj, cfg.dtype)
        progress(f"config {cfg.index} key {j}: {len(qs)} selecting queries checked")


def _progression_on_device(L, k, head, dev, rows_out, lists_out):
    """Fill rows_out [L, k] and lists_out [L*k] (views into the flat index tensors); return col [L+1]."""
    base, gg, ginv = wl.progression_params(L, seed=0, head=head)
    tb, tg = torch.from_numpy(base).to(dev), torch.from_numpy(gg).to(dev)
    t = torch.arange(k, dtype=torch.int64, device=dev)[None, :]
    step = max(1, (1 << 28) // k)                      # about 2 GB of int64 per chunk
    for lo in range(0, L, step):
        hi = min(lo + step, L)
        v = (tb[lo:hi, None] + t * tg[lo:hi, None]) & (L - 1)
        rows_out[lo:hi] = torch.sort(v, dim=1).values.to(torch.int32)
    # key-major lists in closed form: query i holds key j  <=>  ((j - base_i) * ginv_i mod L) < k
    tinv = torch.from_numpy(ginv).to(dev)
    counts = torch.empty(L, dtype=torch.int64, device=dev)
    kstep = max(1, (1 << 28) // L)
    pos = 0
    for lo in range(0, L, kstep):
        hi = min(lo + kstep, L)
        keys = torch.arange(lo, hi, dtype=torch.int64, device=dev)[:, None]
        member = (((keys - tb[None, :]) * tinv[None, :]) & (L - 1)) < k
        counts[lo:hi] = member.sum(dim=1)
        q = torch.nonzero(member)[:, 1].to(torch.int32)     # row-major nonzero: keys ascending, queries ascending
        lists_out[pos:pos + q.numel()] = q
        pos += q.numel()
        del member, q
    assert pos == L * k
    col = torch.zeros(L + 1, dtype=torch.int64, device=dev)
    col[1:] = torch.cumsum(counts, 0)
    return col, (base, gg, ginv)


def test_stage2_full_size(data, progress):
    cfg, ks, g, _, _, host = data
    L, dev = cfg.L, "cuda:0"
    off = wl.idx_offsets(1, cfg.H, L, ks)
    p = dsv.Problem(1, cfg.H, L, cfg.d, cfg.r, cfg.dtype, ks, cfg.scale, sorted_index=True)
    idx = torch.empty(int(off[-1]), dtype=torch.int32, device=dev)
    idx_t = torch.empty(int(off[-1]), dtype=torch.int32, device=dev)
    col = torch.empty((cfg.H, L + 1), dtype=torch.int64, device=dev)
    params = {}
    for h in range(cfg.H):
        col[h], params[h] = _progression_on_device(L, ks[h], h, dev, idx[off[h]:off[h + 1]].view(L, ks[h]),
                                                   idx_t[off[h]:off[h + 1]])
    progress(f"config {cfg.index}: index sets built")
    torch.cuda.empty_cache()
    O, lse = dsv.sparse_attn_fwd(p, g["Q"], g["K"], g["V"], idx)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    dQ, dK, dV = dsv.sparse_attn_bwd_t(p, g["Q"], g["K"], g["V"], idx, idx_t, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    rng = np.random.default_rng(1)
    for h in _host_heads(cfg):
        t, k = host[h], ks[h]
        rows = np.unique(np.concatenate([rng.integers(0, L, size=N_ROWS), [0, L - 1]]))
        idx_rows = wl.progression_idx_rows(L, k, rows, params[h])
        mine = idx[off[h]:off[h + 1]].view(L, k)[torch.from_numpy(rows).cuda()].cpu().numpy()
        assert np.array_equal(idx_rows, mine)     # the test's own two constructions agree
        O_ref, lse_ref = oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], idx_rows, cfg.scale)
        dQ_ref = oracle.sparse_bwd_dq_rows(t["Q"][rows], t["K"], t["V"], idx_rows, t["dO"][rows], cfg.scale)
        sel = torch.from_numpy(rows).cuda()
        assert_close(f"O[h={h}]", O[0, h][sel], O_ref, cfg.dtype)
        assert_close(f"lse[h={h}]", lse[0, h][sel], lse_ref, "f32")
        assert_close(f"dQ[h={h}]", dQ[0, h][sel], dQ_ref, cfg.dtype)
    h = _host_heads(cfg)[0]
    t, k = host[h], ks[h]
    for j in rng.integers(0, L, size=N_KEYS - 1).tolist() + [L - 1]:
        qs = wl.progression_queries_of_key(L, k, j, params[h])
        mine = idx_t[off[h] + int(col[h, j]):off[h] + int(col[h, j + 1])].cpu().numpy().astype(np.int64)
        assert np.array_equal(qs, mine)
        idx_sel = wl.progression_idx_rows(L, k, qs, params[h])
        dKj, dVj = oracle.sparse_bwd_dkdv_key(j, t["Q"][qs], t["dO"][qs], idx_sel, t["K"], t["V"], cfg.scale)
        assert_close(f"dK[h={h}, j={j}]", dK[0, h, j], dKj, cfg.dtype)
        assert_close(f"dV[h={h}, j={j}]", dV[0, h, j], dVj, cfg.dtype)
        progress(f"config {cfg.index} key {j}: {len(qs)} selecting queries checked")


GROUPED_CONFIGS = (1, 2)     # config 2 is the shape bench.py --grouped times
CUBE = (2, 2, 2)
N_GROUPS = 24                # sampled groups per checked head (plus the first and the last)


def test_grouped_full_size(data, progress):
    """The query-grouped variant at full size, in the launch configuration bench.py --grouped times (sorted-index flag:
    the L2-blocked grouped kernels): stage 1 on the groups' centre queries, grouped forward and backward on the index it
    wrote.  Sampled groups: the group's row against the oracle's selection on the device's own score bits of the centre
    query (bit-exact), then O, lse, dQ of all its members against the oracle with that row; sampled keys: the key's list
    of groups against the column of the group index, then dK, dV against the oracle's per-key routine over the members
    of the selecting groups."""
    cfg, ks, g, Wq, Wk, host = data
    if cfg.index not in GROUPED_CONFIGS:
        pytest.skip("grouped full-size check runs at configs 1 and 2")
    L, G = cfg.L, CUBE[0] * CUBE[1] * CUBE[2]
    Lq = L // G
    grp = dsv.Grouping(cfg.grid, CUBE)
    p = dsv.Problem(1, cfg.H, L, cfg.d, cfg.r, cfg.dtype, ks, cfg.scale, sorted_index=True)
    off = np.concatenate([[0], np.cumsum([Lq * k for k in ks])]).astype(np.int64)
    idx_g, idx_t_g, col = dsv.lowrank_topk_grouped(p, grp, g["Q"], g["K"], Wq, Wk)
    Qlr, Klr = dsv.lowrank_project(p, g["Q"], g["K"], Wq, Wk)
    torch.cuda.synchronize()
    progress(f"config {cfg.index} grouped: stage 1 done")
    tokens = oracle.group_tokens(cfg.grid, CUBE)            # [Lq, G] token ids of every group's members
    centre = tokens[:, oracle.group_centre(CUBE)]

    def rows_of(h):
        return idx_g[off[h]:off[h + 1]].view(Lq, ks[h])

    for h in range(cfg.H):
        part = rows_of(h)
        assert int(part.min()) >= 0 and int(part.max()) < L
        assert bool((part[:, 1:] > part[:, :-1]).all()), f"head {h}: group rows not strictly ascending"
        assert int(col[h, 0]) == 0 and int(col[h, -1]) == Lq * ks[h]
    rng = np.random.default_rng(1)
    sampled = {}
    for h in _host_heads(cfg):
        groups = np.unique(np.concatenate([rng.integers(0, Lq, size=N_GROUPS), [0, Lq - 1]])).astype(np.int64)
        S_gpu = dsv.lowrank_scores_rows(p, Qlr, Klr, 0, h, torch.from_numpy(centre[groups].astype(np.int32)).cuda())
        torch.cuda.synchronize()
        got = rows_of(h)[torch.from_numpy(groups).cuda()].cpu().numpy()
        want = oracle.topk_from_scores(S_gpu.cpu().numpy().astype(np.float64), ks[h])
        assert np.array_equal(want, got), f"head {h}: a group's row is not its centre query's selection"
        sampled[h] = (groups, got)
    del Qlr, Klr
    torch.cuda.empty_cache()

    O, lse = dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], idx_g)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    dQ, dK, dV = dsv.sparse_attn_bwd_grouped(p, grp, g["Q"], g["K"], g["V"], idx_g, idx_t_g, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    torch.cuda.empty_cache()
    progress(f"config {cfg.index} grouped: stage 2 done")
    for h in _host_heads(cfg):
        t = host[h]
        groups, rows_g = sampled[h]
        rows = tokens[groups].reshape(-1).astype(np.int64)            # all members of the sampled groups
        idx_rows = np.repeat(rows_g, G, axis=0)                       # every member attends its group's row
        O_ref, lse_ref = oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], idx_rows, cfg.scale)
        dQ_ref = oracle.sparse_bwd_dq_rows(t["Q"][rows], t["K"], t["V"], idx_rows, t["dO"][rows], cfg.scale)
        sel = torch.from_numpy(rows).cuda()
        assert_close(f"grouped O[h={h}]", O[0, h][sel], O_ref, cfg.dtype)
        assert_close(f"grouped lse[h={h}]", lse[0, h][sel], lse_ref, "f32")
        assert_close(f"grouped dQ[h={h}]", dQ[0, h][sel], dQ_ref, cfg.dtype)
    progress(f"config {cfg.index} grouped: O, lse, dQ of {len(rows)} member rows per checked head match")
    h = _host_heads(cfg)[0]
    t, k, rows_dev = host[h], ks[h], rows_of(h)
    lens = (col[h, 1:] - col[h, :-1]).cpu().numpy()
    capped = np.where(lens * G <= MAX_LIST, lens, -1)
    keys = [int(capped.argmax()), int(lens.argmin())] + rng.integers(0, L, size=4).tolist()
    for j in keys:
        gs_dev = _column_of(rows_dev, j, Lq, k)
        mine = idx_t_g[off[h] + int(col[h, j]):off[h] + int(col[h, j + 1])]
        assert torch.equal(gs_dev.to(torch.int32), mine), f"key {j}: idx_t_g list is not the column of idx_g"
        gs = gs_dev.cpu().numpy()
        dKj, dVj = np.zeros(cfg.d), np.zeros(cfg.d)
        step = max(1, (1 << 27) // (k * G))
        for lo in range(0, len(gs), step):
            part = gs[lo:lo + step]
            members = tokens[part].reshape(-1).astype(np.int64)
            idx_sel = np.repeat(rows_dev[gs_dev[lo:lo + step]].cpu().numpy(), G, axis=0)
            a, b = oracle.sparse_bwd_dkdv_key(j, t["Q"][members], t["dO"][members], idx_sel, t["K"], t["V"], cfg.scale)
            dKj += a
            dVj += b
        if len(gs) == 0:
            assert float(dK[0, h, j].abs().max()) == 0.0 and float(dV[0, h, j].abs().max()) == 0.0
        assert_close(f"grouped dK[h={h}, j={j}]", dK[0, h, j], dKj, cfg.dtype)
        assert_close(f"grouped dV[h={h}, j={j}]", dV[0, h, j], dVj, cfg.dtype)
        progress(f"config {cfg.index} grouped key {j}: {len(gs)} selecting groups checked")
