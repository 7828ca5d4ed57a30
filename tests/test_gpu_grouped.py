"""GPU parity of the query-grouped variant (dsv_lowrank_topk_grouped, dsv_sparse_attn_fwd_grouped,
dsv_sparse_attn_bwd_grouped) against the CPU oracle's grouped routines, through the C ABI.

Selection: bit-exact on exact-arithmetic (ternary) inputs; on Gaussian inputs a group's row must equal
the per-query device selection of its centre query (same score bits), whose own parity the stage-1 tests
establish.  Attention: O, lse, dQ, dK, dV element-wise within the stage-2 tolerance, on the ORACLE's index.
"""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import assert_close
from workloads.configs import WorkloadConfig

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def _cfg(grid, d=128, r=16, dtype="bf16", R=32, H=2):
    return WorkloadConfig(index=300, name="grouped_gpu", B=1, H=H, grid=grid, d=d, r=r, k=None, k_choices=(),
                          dtype=dtype, basis_rank=R, scale=2.0 / math.sqrt(d))


def _numpy_group_tokens(grid, cube):
    F, H, W = grid
    gf, gh, gw = cube
    t = np.arange(F * H * W).reshape(F // gf, gf, H // gh, gh, W // gw, gw).transpose(0, 2, 4, 1, 3, 5)
    return t.reshape(-1, gf * gh * gw)


def _dev(a, td):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()


@pytest.mark.parametrize("grid,cube,ks,dtype,d,r", [((4, 8, 16), (2, 2, 2), [100, 33], "bf16", 128, 16),
                                                    ((2, 6, 10), (1, 3, 2), [120, 1], "f32", 64, 32),
                                                    ((3, 5, 7), (1, 1, 1), [17, 50], "bf16", 64, 16)])
def test_grouped_selection_bit_exact_on_ternary_inputs(grid, cube, ks, dtype, d, r):
    L, H = grid[0] * grid[1] * grid[2], len(ks)
    G = cube[0] * cube[1] * cube[2]
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    Qs, Ks, Wqs, Wks = zip(*(wl.ternary_head_tensors(L, d, r, seed=5, head=h) for h in range(H)))
    p = dsv.Problem(1, H, L, d, r, dtype, ks, 1.0)
    g = dsv.Grouping(grid, cube)
    idx_g, idx_t_g, col = dsv.lowrank_topk_grouped(p, g, _dev(np.stack(Qs), td)[None], _dev(np.stack(Ks), td)[None],
                                                   _dev(np.stack(Wqs), td), _dev(np.stack(Wks), td))
    torch.cuda.synchronize()
    idx_g, idx_t_g, col = idx_g.cpu().numpy(), idx_t_g.cpu().numpy(), col.cpu().numpy()
    off = wl.idx_offsets(1, H, L // G, ks)
    for h in range(H):
        ref = oracle.lowrank_topk_grouped(Qs[h], Ks[h], Wqs[h], Wks[h], grid, cube, ks[h], dtype)
        rows = idx_g[off[h]:off[h + 1]].reshape(L // G, ks[h])
        assert np.array_equal(rows, ref), f"head {h}"
        # key-major lists: the exact transpose, groups ascending
        counts = np.bincount(rows.reshape(-1), minlength=L)
        assert col[h, 0] == 0 and np.array_equal(np.diff(col[h]), counts)
        order = np.argsort(rows.reshape(-1), kind="stable")
        assert np.array_equal(idx_t_g[off[h]:off[h + 1]], np.repeat(np.arange(L // G, dtype=np.int32), ks[h])[order])


def test_grouped_selection_is_the_centre_querys_device_selection():
    cfg = _cfg((4, 16, 32), H=2)
    cube, ks = (2, 2, 2), [200, 64]
    L = cfg.L
    td = torch.bfloat16
    t = [wl.head_tensors(cfg, h, names=("Q", "K")) for h in range(2)]
    W = [wl.predictor_weights(cfg, h) for h in range(2)]
    Q, K = _dev(np.stack([x["Q"] for x in t]), td)[None], _dev(np.stack([x["K"] for x in t]), td)[None]
    Wq, Wk = _dev(np.stack([w[0] for w in W]), td), _dev(np.stack([w[1] for w in W]), td)
    p = dsv.Problem(1, 2, L, cfg.d, cfg.r, "bf16", ks, cfg.scale)
    idx_q = dsv.lowrank_topk(p, Q, K, Wq, Wk).cpu().numpy()
    idx_g, _, _ = dsv.lowrank_topk_grouped(p, dsv.Grouping(cfg.grid, cube), Q, K, Wq, Wk, transposed=False)
    idx_g = idx_g.cpu().numpy()
    centre = _numpy_group_tokens(cfg.grid, cube)[:, oracle.group_centre(cube)]
    off_q, off_g = wl.idx_offsets(1, 2, L, ks), wl.idx_offsets(1, 2, L // 8, ks)
    for h in range(2):
        assert np.array_equal(idx_g[off_g[h]:off_g[h + 1]].reshape(L // 8, ks[h]),
                              idx_q[off_q[h]:off_q[h + 1]].reshape(L, ks[h])[centre])


CASES = [((4, 8, 16), (2, 2, 2), [100, 33]),      # G = 8, ragged tails (100 = 3 * 32 + 4), k < 32 ... > 32
         ((2, 6, 10), (1, 3, 2), [120, 1]),       # G = 6; k = L (dense limit) and k = 1
         ((3, 5, 7), (1, 1, 1), [17, 50]),        # G = 1: the per-query problem
         ((8, 32, 32), (2, 2, 2), [512, 300])]    # L = 8192: many tiles per row, many groups per key


@pytest.fixture(scope="module", params=CASES, ids=lambda c: f"grid{c[0]}_cube{c[1]}")
def case(request):
    grid, cube, ks = request.param
    cfg = _cfg(grid, H=len(ks))
    L, H = cfg.L, cfg.H
    G = cube[0] * cube[1] * cube[2]
    td = torch.bfloat16
    t = [wl.head_tensors(cfg, h) for h in range(H)]
    g = {n: _dev(np.stack([x[n] for x in t]), td)[None] for n in ("Q", "K", "V", "dO")}
    idx_g = [wl.random_subset_idx(L, k, L // G, seed=7, head=h) for h, k in enumerate(ks)]      # the oracle side's rows
    return cfg, cube, ks, t, g, idx_g


@pytest.mark.parametrize("blocked", [False, True], ids=["plain", "l2_blocked"])
def test_grouped_forward_matches_oracle(case, blocked):
    cfg, cube, ks, t, g, idx_g = case
    p = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, "bf16", ks, cfg.scale, sorted_index=blocked)
    assert (dsv.sparse_attn_fwd_grouped_workspace(p, dsv.Grouping(cfg.grid, cube)) > 0) == blocked
    grp = dsv.Grouping(cfg.grid, cube)
    flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in idx_g])).cuda()
    O, lse = dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat)
    torch.cuda.synchronize()
    for h in range(cfg.H):
        O_ref, lse_ref = oracle.sparse_fwd_grouped(t[h]["Q"], t[h]["K"], t[h]["V"], idx_g[h], cfg.grid, cube, cfg.scale)
        assert_close(f"O[h={h}]", O[0, h], O_ref, "bf16")
        assert_close(f"lse[h={h}]", lse[0, h], lse_ref, "f32")
    if ks[0] == cfg.L:   # dense limit
        O_d, lse_d = oracle.dense_fwd(t[0]["Q"], t[0]["K"], t[0]["V"], cfg.scale)
        assert_close("O vs dense", O[0, 0], O_d, "bf16")


@pytest.mark.parametrize("blocked", [False, True], ids=["plain", "l2_blocked"])
def test_grouped_backward_matches_oracle(case, blocked):
    cfg, cube, ks, t, g, idx_g = case
    L, G = cfg.L, cube[0] * cube[1] * cube[2]
    p = dsv.Problem(1, cfg.H, L, cfg.d, cfg.r, "bf16", ks, cfg.scale, sorted_index=blocked)
    grp = dsv.Grouping(cfg.grid, cube)
    flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in idx_g])).cuda()
    # key-major lists of groups, ascending: a stable sort of the (group, key) pairs by key, written out here
    lists, cols = [], []
    for h, k in enumerate(ks):
        order = np.argsort(idx_g[h].reshape(-1), kind="stable")
        lists.append(np.repeat(np.arange(L // G, dtype=np.int32), k)[order])
        cols.append(np.concatenate([[0], np.cumsum(np.bincount(idx_g[h].reshape(-1), minlength=L))]).astype(np.int64))
    idx_t_g = torch.from_numpy(np.concatenate(lists)).cuda()
    col = torch.from_numpy(np.stack(cols)).cuda()
    O, lse = dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat)
    dQ, dK, dV = dsv.sparse_attn_bwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat, idx_t_g, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    for h in range(cfg.H):
        dQ_ref, dK_ref, dV_ref = oracle.sparse_bwd_grouped(t[h]["Q"], t[h]["K"], t[h]["V"], idx_g[h], t[h]["dO"], cfg.grid,
                                                           cube, cfg.scale)
        assert_close(f"dQ[h={h}]", dQ[0, h], dQ_ref, "bf16")
        assert_close(f"dK[h={h}]", dK[0, h], dK_ref, "bf16")
        assert_close(f"dV[h={h}]", dV[0, h], dV_ref, "bf16")
        unselected = np.bincount(idx_g[h].reshape(-1), minlength=L) == 0
        if unselected.any():
            assert float(dK[0, h][torch.from_numpy(unselected).cuda()].abs().max()) == 0.0


@pytest.mark.parametrize("grid,cube,k", [((2, 4, 6), (1, 1, 2), 31), ((3, 4, 6), (3, 1, 1), 32), ((2, 4, 8), (1, 2, 2), 33),
                                         ((5, 2, 6), (5, 1, 1), 1), ((2, 7, 6), (1, 7, 1), 63), ((4, 4, 4), (2, 2, 2), 64),
                                         ((2, 8, 8), (2, 2, 2), 65), ((2, 4, 8), (1, 1, 4), 64),
                                         ((4, 8, 8), (2, 4, 4), 40), ((2, 4, 6), (2, 2, 3), 33), ((4, 4, 8), (4, 2, 2), 128),
                                         ((2, 6, 10), (1, 3, 5), 31), ((8, 8, 8), (2, 4, 4), 200)])
@pytest.mark.parametrize("blocked", [False, True], ids=["plain", "l2_blocked"])
def test_every_group_size_and_tile_boundary(grid, cube, k, blocked):
    """G = 2, 3, 4, 5, 7, 8 (four groups per block) and 12, 15, 16, 32 (one group per block, its waves sharing the
    gathered rows) with k just below, at and just above whole 32-key tiles: forward and backward against the grouped
    oracle (one head, the oracle's index)."""
    cfg = _cfg(grid, H=1)
    L, G = cfg.L, cube[0] * cube[1] * cube[2]
    t = wl.head_tensors(cfg, 0)
    g = {n: _dev(t[n][None], torch.bfloat16)[None] for n in ("Q", "K", "V", "dO")}
    idx_g = wl.random_subset_idx(L, k, L // G, seed=11, head=0)
    p = dsv.Problem(1, 1, L, cfg.d, cfg.r, "bf16", [k], cfg.scale, sorted_index=blocked)
    grp = dsv.Grouping(cfg.grid, cube)
    flat = torch.from_numpy(idx_g.reshape(-1)).cuda()
    order = np.argsort(idx_g.reshape(-1), kind="stable")
    idx_t_g = torch.from_numpy(np.repeat(np.arange(L // G, dtype=np.int32), k)[order]).cuda()
    col = torch.from_numpy(np.concatenate([[0], np.cumsum(np.bincount(idx_g.reshape(-1), minlength=L))]).astype(np.int64)[None]).cuda()
    O, lse = dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat)
    dQ, dK, dV = dsv.sparse_attn_bwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat, idx_t_g, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    O_ref, lse_ref = oracle.sparse_fwd_grouped(t["Q"], t["K"], t["V"], idx_g, cfg.grid, cube, cfg.scale)
    dQ_ref, dK_ref, dV_ref = oracle.sparse_bwd_grouped(t["Q"], t["K"], t["V"], idx_g, t["dO"], cfg.grid, cube, cfg.scale)
    for name, got, ref, dt in (("O", O, O_ref, "bf16"), ("lse", lse, lse_ref, "f32"), ("dQ", dQ, dQ_ref, "bf16"),
                               ("dK", dK, dK_ref, "bf16"), ("dV", dV, dV_ref, "bf16")):
        assert_close(f"{name} G={G} k={k}", got[0, 0], ref, dt)


def test_grouped_arguments_are_checked_on_the_host():
    import ctypes
    lib = dsv.load_library()
    one = ctypes.c_void_p(256)
    p = dsv.Problem(1, 1, 512, 128, 16, "bf16", [32], 0.1)
    bad_grid = dsv.Grouping((4, 8, 15), (2, 2, 1))        # 480 tokens, not L
    no_tiling = dsv.Grouping((4, 8, 16), (2, 3, 2))        # 3 does not divide 8
    for gg in (bad_grid, no_tiling):
        assert lib.dsv_sparse_attn_fwd_grouped(p.c, gg.c, one, one, one, one, one, one, None, 0, None) == -1
        assert dsv.lowrank_topk_grouped_workspace(p, gg) == 0
    huge = dsv.Grouping((8, 8, 8), (8, 4, 4))              # G = 128: beyond the largest group accepted (64)
    assert lib.dsv_sparse_attn_fwd_grouped(p.c, huge.c, one, one, one, one, one, one, None, 0, None) == -2
    big = dsv.Grouping((4, 8, 16), (2, 4, 8))              # G = 64 runs through the per-query kernels: needs its workspace
    assert dsv.sparse_attn_fwd_grouped_workspace(p, big) > p.nnz * 4
    assert lib.dsv_sparse_attn_fwd_grouped(p.c, big.c, one, one, one, one, one, one, None, 0, None) == -3


@pytest.mark.parametrize("dtype,d,grid,cube,ks", [("f32", 64, (4, 8, 8), (2, 2, 2), [40, 7]),       # fp32, d = 64
                                                  ("bf16", 128, (4, 8, 16), (2, 4, 8), [100, 33]),  # G = 64
                                                  ("bf16", 64, (4, 4, 8), (1, 2, 2), [128, 20]),    # d = 64; k = L
                                                  ("f32", 128, (2, 6, 6), (2, 3, 3), [9, 72])])     # G = 18, fp32, k = L
@pytest.mark.parametrize("sorted_index", [False, True], ids=["plain", "l2_blocked"])
def test_general_grouped_path_matches_oracle(dtype, d, grid, cube, ks, sorted_index):
    """dtypes, head dimensions and cube sizes the group kernels proper do not cover run the per-query kernels on
    queries reordered group by group with the group index expanded: same contract, checked the same way."""
    cfg = _cfg(grid, d=d, dtype=dtype, H=len(ks))
    L, G = cfg.L, cube[0] * cube[1] * cube[2]
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    t = [wl.head_tensors(cfg, h) for h in range(cfg.H)]
    g = {n: _dev(np.stack([x[n] for x in t]), td)[None] for n in ("Q", "K", "V", "dO")}
    idx_g = [wl.random_subset_idx(L, k, L // G, seed=3, head=h) for h, k in enumerate(ks)]
    p = dsv.Problem(1, cfg.H, L, d, cfg.r, dtype, ks, cfg.scale, sorted_index=sorted_index)
    grp = dsv.Grouping(cfg.grid, cube)
    flat = torch.from_numpy(np.concatenate([x.reshape(-1) for x in idx_g])).cuda()
    lists, cols = [], []
    for h, k in enumerate(ks):
        order = np.argsort(idx_g[h].reshape(-1), kind="stable")
        lists.append(np.repeat(np.arange(L // G, dtype=np.int32), k)[order])
        cols.append(np.concatenate([[0], np.cumsum(np.bincount(idx_g[h].reshape(-1), minlength=L))]).astype(np.int64))
    idx_t_g = torch.from_numpy(np.concatenate(lists)).cuda()
    col = torch.from_numpy(np.stack(cols)).cuda()
    O, lse = dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat)
    dQ, dK, dV = dsv.sparse_attn_bwd_grouped(p, grp, g["Q"], g["K"], g["V"], flat, idx_t_g, col, O, lse, g["dO"])
    torch.cuda.synchronize()
    for h in range(cfg.H):
        O_ref, lse_ref = oracle.sparse_fwd_grouped(t[h]["Q"], t[h]["K"], t[h]["V"], idx_g[h], cfg.grid, cube, cfg.scale)
        dQ_ref, dK_ref, dV_ref = oracle.sparse_bwd_grouped(t[h]["Q"], t[h]["K"], t[h]["V"], idx_g[h], t[h]["dO"], cfg.grid, cube,
                                                           cfg.scale)
        for name, got, ref, dt in (("O", O, O_ref, dtype), ("lse", lse, lse_ref, "f32"), ("dQ", dQ, dQ_ref, dtype),
                                   ("dK", dK, dK_ref, dtype), ("dV", dV, dV_ref, dtype)):
            assert_close(f"{name}[h={h}] {dtype} d={d} G={G}", got[0, h], ref, dt)


def test_group_overlap_and_the_choice_of_the_group_size():
    """dsv_group_overlap against the oracle (the counts behind both are integers: equal up to the final float
    division) on rows in no particular order and on a real selection of smooth inputs; dsv_choose_grouping picks the
    largest cube that keeps the required share in every head."""
    grid, ks = (4, 8, 8), [37, 200]
    L = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng(9)
    rows = [np.stack([rng.permutation(L)[:k] for _ in range(L)]).astype(np.int32) for k in ks]
    p = dsv.Problem(1, len(ks), L, 128, 16, "bf16", ks, 1.0)
    flat = torch.from_numpy(np.concatenate([r.reshape(-1) for r in rows])).cuda()
    for cube in ((2, 2, 2), (1, 1, 1), (4, 2, 1), (2, 4, 8)):
        got = dsv.group_overlap(p, dsv.Grouping(grid, cube), flat).cpu().numpy()
        want = np.array([oracle.group_overlap(r, grid, cube) for r in rows])
        assert np.allclose(got, want, rtol=0, atol=1e-6), (cube, got, want)
        assert np.array_equal(np.rint(got.astype(np.float64) * L * np.array(ks)), np.rint(want * L * np.array(ks)))
    # a real selection: smooth inputs, identity-like predictor (W = basis^T): neighbouring queries share most keys
    cfg = _cfg((8, 8, 16), d=128, r=32, R=32, H=1)
    t = wl.head_tensors_smooth(cfg, 0, sigma=5.0, names=("Q", "K"))
    W = wl.basis(cfg, 0).T.astype(np.float32).copy()
    k = cfg.L // 16
    ps = dsv.Problem(1, 1, cfg.L, cfg.d, cfg.r, "bf16", [k], cfg.scale)
    dev = lambda a: _dev(a, torch.bfloat16)
    idx = dsv.lowrank_topk(ps, dev(t["Q"][None])[None], dev(t["K"][None])[None], dev(W[None]), dev(W[None]))
    torch.cuda.synchronize()
    rows_s = idx.view(cfg.L, k).cpu().numpy()
    cubes = [(1, 1, 1), (2, 2, 2), (1, 2, 2), (4, 4, 4), (3, 2, 2), (8, 8, 16)]       # (3, 2, 2) does not tile; the last has G > 64
    chosen, ov = dsv.choose_grouping(ps, cfg.grid, cubes, idx, min_overlap=0.8)
    for c, cube in enumerate(cubes):
        if cfg.grid[0] % cube[0] or cube[0] * cube[1] * cube[2] > 64:
            assert ov[c][0] == -1.0
        else:
            assert abs(ov[c][0] - oracle.group_overlap(rows_s, cfg.grid, cube)) < 1e-6
    ok = [c for c, cube in enumerate(cubes) if ov[c][0] >= 0.8]
    assert chosen == max(ok, key=lambda c: cubes[c][0] * cubes[c][1] * cubes[c][2])
    assert ov[0][0] == 1.0 and chosen != 0            # the unit cube always qualifies; on smooth inputs a larger one does too
    assert dsv.choose_grouping(ps, cfg.grid, cubes[1:2], idx, min_overlap=1.01)[0] == -1
