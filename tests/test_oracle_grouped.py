"""Pins of the oracle's query-grouping routines (paper Sec. "Sparse Attention with Query Grouping",
Observation 5), none of which needs a GPU:
  * the token <-> cube map against a plain numpy construction of the grid, and the centre voxel;
  * a cube of 1 x 1 x 1 is the per-query path, bit for bit;
  * a group whose members hold identical queries gets what per-query selection gives each member;
  * grouped attention equals the per-query routines on the expanded index (additivity of dK, dV over the
    members), the dense limit at k = L, central finite differences with the shared rows held fixed;
  * on spatially smooth inputs neighbouring queries share most of their top keys (the paper reports
    about 80 % inside 2 x 2 x 2 cubes), on the i.i.d. inputs they do not.
"""
import numpy as np
import pytest

import oracle
import workloads as wl
from workloads.configs import WorkloadConfig


def _cfg(grid, d=64, r=16, dtype="f32", R=32, index=200):
    return WorkloadConfig(index=index, name="grouped_case", B=1, H=1, grid=grid, d=d, r=r, k=None, k_choices=(),
                          dtype=dtype, basis_rank=R, scale=1.0 / np.sqrt(d))


def _numpy_group_tokens(grid, cube):
    F, H, W = grid
    gf, gh, gw = cube
    tok = np.arange(F * H * W).reshape(F, H, W)
    t = tok.reshape(F // gf, gf, H // gh, gh, W // gw, gw).transpose(0, 2, 4, 1, 3, 5)
    return t.reshape(-1, gf * gh * gw)


@pytest.mark.parametrize("grid,cube", [((4, 4, 8), (2, 2, 2)), ((2, 6, 4), (1, 3, 2)), ((8, 8, 16), (2, 2, 4)),
                                       ((3, 2, 5), (1, 1, 1)), ((4, 4, 4), (4, 2, 1))])
def test_group_map_matches_a_numpy_tiling_of_the_grid(grid, cube):
    got = oracle.group_tokens(grid, cube)
    want = _numpy_group_tokens(grid, cube)
    assert np.array_equal(got, want)
    assert np.array_equal(np.sort(got.reshape(-1)), np.arange(grid[0] * grid[1] * grid[2]))   # a partition of the tokens
    # the centre voxel: offset side // 2 along every axis
    c = oracle.group_centre(cube)
    assert c == ((cube[0] // 2) * cube[1] + cube[1] // 2) * cube[2] + cube[2] // 2
    f0, h0, w0 = np.unravel_index(want[0, c], grid)
    assert (f0, h0, w0) == (cube[0] // 2, cube[1] // 2, cube[2] // 2)


def test_cube_sizes_must_divide_the_grid():
    assert oracle.group_member(0, 0, (4, 4, 6), (2, 2, 4)) == -1


def test_unit_cube_is_the_per_query_path_bit_for_bit():
    cfg = _cfg((4, 4, 8))
    t = wl.head_tensors(cfg, 0)
    Wq, Wk = wl.predictor_weights(cfg, 0)
    k = 19
    idx = oracle.lowrank_topk(t["Q"], t["K"], Wq, Wk, k, cfg.dtype)
    idx_g = oracle.lowrank_topk_grouped(t["Q"], t["K"], Wq, Wk, cfg.grid, (1, 1, 1), k, cfg.dtype)
    assert np.array_equal(idx, idx_g)
    O, lse = oracle.sparse_fwd(t["Q"], t["K"], t["V"], idx, cfg.scale)
    Og, lseg = oracle.sparse_fwd_grouped(t["Q"], t["K"], t["V"], idx_g, cfg.grid, (1, 1, 1), cfg.scale)
    assert np.array_equal(O, Og) and np.array_equal(lse, lseg)
    for a, b in zip(oracle.sparse_bwd(t["Q"], t["K"], t["V"], idx, t["dO"], cfg.scale),
                    oracle.sparse_bwd_grouped(t["Q"], t["K"], t["V"], idx_g, t["dO"], cfg.grid, (1, 1, 1), cfg.scale)):
        assert np.array_equal(a, b)


def test_selection_is_the_centre_querys_and_identical_members_lose_nothing():
    cfg = _cfg((4, 4, 8))
    cube = (2, 2, 2)
    t = wl.head_tensors(cfg, 0)
    Wq, Wk = wl.predictor_weights(cfg, 0)
    k = 25
    tokens = _numpy_group_tokens(cfg.grid, cube)
    centre = tokens[:, oracle.group_centre(cube)]
    idx_q = oracle.lowrank_topk(t["Q"], t["K"], Wq, Wk, k, cfg.dtype)
    idx_g = oracle.lowrank_topk_grouped(t["Q"], t["K"], Wq, Wk, cfg.grid, cube, k, cfg.dtype)
    assert np.array_equal(idx_g, idx_q[centre])                 # the proxy is the centre query, nobody else
    assert not np.array_equal(idx_g, idx_q[tokens[:, 0]])
    # every member a copy of its group's centre query: grouping changes nothing for any member
    Q2 = t["Q"].copy()
    Q2[tokens.reshape(-1)] = np.repeat(t["Q"][centre], tokens.shape[1], axis=0)
    idx_q2 = oracle.lowrank_topk(Q2, t["K"], Wq, Wk, k, cfg.dtype)
    idx_g2 = oracle.lowrank_topk_grouped(Q2, t["K"], Wq, Wk, cfg.grid, cube, k, cfg.dtype)
    assert np.array_equal(oracle.group_expand_idx(idx_g2, cfg.grid, cube), idx_q2)


def test_grouped_attention_is_per_query_attention_over_the_shared_row():
    cfg = _cfg((2, 4, 8))
    cube = (2, 2, 2)
    L = cfg.L
    t = wl.head_tensors(cfg, 0)
    Wq, Wk = wl.predictor_weights(cfg, 0)
    k = 11
    idx_g = oracle.lowrank_topk_grouped(t["Q"], t["K"], Wq, Wk, cfg.grid, cube, k, cfg.dtype)
    tokens = _numpy_group_tokens(cfg.grid, cube)
    idx = np.empty((L, k), dtype=np.int32)                       # expansion written out independently of the C routine
    for g in range(tokens.shape[0]):
        idx[tokens[g]] = idx_g[g]
    assert np.array_equal(idx, oracle.group_expand_idx(idx_g, cfg.grid, cube))
    O, lse = oracle.sparse_fwd(t["Q"], t["K"], t["V"], idx, cfg.scale)
    Og, lseg = oracle.sparse_fwd_grouped(t["Q"], t["K"], t["V"], idx_g, cfg.grid, cube, cfg.scale)
    assert np.array_equal(O, Og) and np.array_equal(lse, lseg)
    dQ, dK, dV = oracle.sparse_bwd(t["Q"], t["K"], t["V"], idx, t["dO"], cfg.scale)
    dQg, dKg, dVg = oracle.sparse_bwd_grouped(t["Q"], t["K"], t["V"], idx_g, t["dO"], cfg.grid, cube, cfg.scale)
    assert np.array_equal(dQ, dQg) and np.array_equal(dK, dKg) and np.array_equal(dV, dVg)
    # library check: masked dense attention in torch, autograd for the gradients
    import torch
    Qt, Kt, Vt = (torch.tensor(t[n], dtype=torch.float64, requires_grad=True) for n in ("Q", "K", "V"))
    mask = torch.zeros(L, L, dtype=torch.bool)
    mask[torch.arange(L)[:, None], torch.from_numpy(idx.astype(np.int64))] = True
    Ot = torch.nn.functional.scaled_dot_product_attention(Qt[None], Kt[None], Vt[None], attn_mask=mask[None], scale=cfg.scale)[0]
    Ot.backward(torch.tensor(t["dO"], dtype=torch.float64))
    assert np.abs(Ot.detach().numpy() - Og).max() < 1e-12
    for ref, got in ((Qt.grad, dQg), (Kt.grad, dKg), (Vt.grad, dVg)):
        assert np.abs(ref.numpy() - got).max() < 1e-11


def test_grouped_dense_limit_and_finite_differences():
    cfg = _cfg((2, 2, 4), d=64)
    cube = (1, 2, 2)
    L = cfg.L
    t = wl.head_tensors(cfg, 0)
    full = np.tile(np.arange(L, dtype=np.int32), (L // 4, 1))
    Og, lseg = oracle.sparse_fwd_grouped(t["Q"], t["K"], t["V"], full, cfg.grid, cube, cfg.scale)
    Od, lsed = oracle.dense_fwd(t["Q"], t["K"], t["V"], cfg.scale)
    assert np.abs(Og - Od).max() < 1e-13 and np.abs(lseg - lsed).max() < 1e-13
    # finite differences of sum(O * dO) with the shared rows held fixed
    idx_g = wl.random_subset_idx(L, 5, L // 4, seed=4)
    dQ, dK, dV = oracle.sparse_bwd_grouped(t["Q"], t["K"], t["V"], idx_g, t["dO"], cfg.grid, cube, cfg.scale)
    def f(Q, K, V):
        O, _ = oracle.sparse_fwd_grouped(Q, K, V, idx_g, cfg.grid, cube, cfg.scale)
        return float((O * t["dO"]).sum())
    rng = np.random.default_rng(0)
    eps = 2.0 ** -10          # exactly representable steps of fp32 inputs
    for name, grad in (("Q", dQ), ("K", dK), ("V", dV)):
        for _ in range(6):
            i, c = int(rng.integers(L)), int(rng.integers(cfg.d))
            plus = {n: t[n].copy() for n in ("Q", "K", "V")}; minus = {n: t[n].copy() for n in ("Q", "K", "V")}
            plus[name][i, c] += eps; minus[name][i, c] -= eps
            fd = (f(plus["Q"], plus["K"], plus["V"]) - f(minus["Q"], minus["K"], minus["V"])) / (2 * eps)
            assert abs(fd - grad[i, c]) < 2e-5 * max(1.0, abs(grad[i, c])), (name, i, c, fd, grad[i, c])


def _overlap_with_centre(idx_q, grid, cube):
    tokens = _numpy_group_tokens(grid, cube)
    centre = tokens[:, oracle.group_centre(cube)]
    k = idx_q.shape[1]
    member = np.zeros((idx_q.shape[0], grid[0] * grid[1] * grid[2]), dtype=bool)
    member[np.arange(idx_q.shape[0])[:, None], idx_q] = True
    shared = (member[tokens] & member[centre][:, None, :]).sum(axis=2)          # [groups, G]
    others = np.arange(tokens.shape[1]) != oracle.group_centre(cube)
    return float(shared[:, others].mean() / k)


def test_neighbouring_queries_share_their_keys_on_smooth_inputs_only():
    cfg = _cfg((8, 8, 16), d=64, r=64, R=32)
    cube = (2, 2, 2)
    k = 64                                                       # 6.25 % of 1024 keys
    eye = np.eye(cfg.d, dtype=np.float32)                         # identity predictor: the exact top-k of Q K^T
    t_iid = wl.head_tensors(cfg, 0, names=("Q", "K"))
    t_sm = wl.head_tensors_smooth(cfg, 0, sigma=5.0, names=("Q", "K"))
    ov_iid = _overlap_with_centre(oracle.lowrank_topk(t_iid["Q"], t_iid["K"], eye, eye, k, "f32"), cfg.grid, cube)
    ov_sm = _overlap_with_centre(oracle.lowrank_topk(t_sm["Q"], t_sm["K"], eye, eye, k, "f32"), cfg.grid, cube)
    assert ov_iid < 0.25, ov_iid          # unrelated queries share about k / L of their keys, plus the common basis
    assert ov_sm > 0.80, ov_sm            # the regime the paper reports for 2 x 2 x 2 cubes (Observation 5)


def test_group_overlap_counts_shared_keys_with_the_centres_row():
    """oracle.group_overlap against plain numpy set intersections, and its closed forms."""
    grid, cube, k = (4, 6, 4), (2, 3, 2), 11
    L = grid[0] * grid[1] * grid[2]
    rng = np.random.default_rng(3)
    idx = np.stack([rng.permutation(L)[:k] for _ in range(L)]).astype(np.int32)      # rows in no particular order
    tokens = _numpy_group_tokens(grid, cube)
    centre = tokens[:, oracle.group_centre(cube)]
    want = sum(len(np.intersect1d(idx[i], idx[centre[g]])) for g in range(tokens.shape[0]) for i in tokens[g])
    assert oracle.group_overlap(idx, grid, cube) == want / (L * k)
    # closed forms: a unit cube keeps everything; identical rows keep everything; rows disjoint from their centre's
    # keep only the centre queries' own share 1 / G
    assert oracle.group_overlap(idx, grid, (1, 1, 1)) == 1.0
    same = np.tile(np.arange(k, dtype=np.int32), (L, 1))
    assert oracle.group_overlap(same, grid, cube) == 1.0
    G = cube[0] * cube[1] * cube[2]
    disjoint = np.tile(np.arange(k, dtype=np.int32), (L, 1))
    disjoint[centre] += k
    assert oracle.group_overlap(disjoint, grid, cube) == 1.0 / G
    # and it agrees with the overlap measured on the smooth inputs above (members other than the centre: (ov G - 1) / (G - 1))
    cfg = _cfg((8, 8, 16), d=64, r=64, R=32)
    eye = np.eye(cfg.d, dtype=np.float32)
    t_sm = wl.head_tensors_smooth(cfg, 0, sigma=5.0, names=("Q", "K"))
    rows = oracle.lowrank_topk(t_sm["Q"], t_sm["K"], eye, eye, 64, "f32")
    ov = oracle.group_overlap(rows, cfg.grid, (2, 2, 2))
    assert abs((ov * 8 - 1) / 7 - _overlap_with_centre(rows, cfg.grid, (2, 2, 2))) < 1e-12
    with pytest.raises(ValueError):
        oracle.group_overlap(idx, grid, (3, 3, 2))
