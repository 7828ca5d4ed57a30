"""GPU parity of stage 1 (dsv_lowrank_project / dsv_lowrank_scores_rows / dsv_lowrank_topk) against
the CPU oracle, through the C ABI.

Bit-exactness of a top-k against a double-precision oracle is only defined when both sides rank
identical score values, so the index sets are checked on three tiers:
  T1  inputs whose scores are exact integers in any summation order -> whole call bit-exact,
      with massive ties exercising "lower index wins";
  T2  the oracle's selection applied to the device's own fp32 score bits -> bit-exact;
  T3  against the pure fp64 oracle: every difference must sit within the fp32 rounding error of
      the threshold score.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import Case, assert_t3_valid, make_cfg, score_error_bound

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def _run_topk(p, Q, K, Wq, Wk):
    idx = dsv.lowrank_topk(p, Q, K, Wq, Wk)
    torch.cuda.synchronize()
    return idx.cpu().numpy()


# ------------------------------------------------------------------------------ projection
@pytest.mark.parametrize("dtype,d,r,L", [("bf16", 128, 16, 300), ("bf16", 64, 32, 129), ("f32", 64, 16, 1024),
                                         ("bf16", 128, 64, 70), ("f32", 128, 32, 65)])
def test_project_matches_oracle(dtype, d, r, L):
    cfg = make_cfg(L, d, r, 2, dtype)
    case = Case(cfg, [1, 1], names=("Q", "K"))
    p = case.problem(dsv)
    Qlr, Klr = dsv.lowrank_project(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    torch.cuda.synchronize()
    for h in range(cfg.H):
        for got, X, W in ((Qlr, case.host["Q"][h], case.Wq[h]), (Klr, case.host["K"][h], case.Wk[h])):
            ref = oracle.project(X, W, dtype).astype(np.float64)
            g = got[0, h].to(torch.float64).cpu().numpy()
            exact = X.astype(np.float64) @ W.astype(np.float64)
            if dtype == "bf16":
                # one bf16 ulp of the result, plus the fp32 accumulation error of the d-term sum (which
                # dominates only when the terms cancel to a tiny result)
                ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.maximum(np.abs(g), np.abs(ref)), 1e-30))) - 7)
                acc_err = d * 2.0 ** -24 * (np.abs(X).astype(np.float64) @ np.abs(W).astype(np.float64))
                assert np.all(np.abs(g - ref) <= ulp * 1.0001 + acc_err)
                assert (g == ref).mean() > 0.98                           # and almost always identical
            else:
                assert np.all(np.abs(g - exact) <= 1e-5 * np.maximum(1.0, np.abs(exact)))


# ------------------------------------------------------------------------------ T1
@pytest.mark.parametrize("dtype,L,d,r,ks", [("bf16", 777, 128, 16, [100, 33]), ("f32", 130, 64, 32, [130, 1]),
                                            ("bf16", 2048, 64, 32, [64, 2047]), ("bf16", 31, 128, 64, [5, 31])])
def test_t1_exact_inputs_whole_call_bit_exact(dtype, L, d, r, ks):
    H = len(ks)
    Qs, Ks, Wqs, Wks = zip(*(wl.ternary_head_tensors(L, d, r, seed=1, head=h) for h in range(H)))
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    dev = lambda a: torch.from_numpy(np.stack(a)).cuda().to(td).contiguous()
    p = dsv.Problem(1, H, L, d, r, dtype, ks, 1.0)
    idx = _run_topk(p, dev(Qs)[None], dev(Ks)[None], dev(Wqs), dev(Wks))
    off = wl.idx_offsets(1, H, L, ks)
    for h in range(H):
        ref = oracle.lowrank_topk(Qs[h], Ks[h], Wqs[h], Wks[h], ks[h], dtype)
        assert np.array_equal(idx[off[h]:off[h + 1]].reshape(L, ks[h]), ref), f"head {h}"


def test_all_equal_scores_take_the_lowest_indices():
    L, d, r, k = 500, 64, 16, 37
    cfg = make_cfg(L, d, r, 1, "bf16")
    case = Case(cfg, [k], names=("Q", "K"))
    p = case.problem(dsv)
    idx = _run_topk(p, torch.zeros_like(case.dev["Q"]), case.dev["K"], case.dWq, case.dWk)
    assert np.array_equal(idx.reshape(L, k), np.tile(np.arange(k, dtype=np.int32), (L, 1)))


# ------------------------------------------------------------------------------ T2 / T3
@pytest.mark.parametrize("which", ["config0", "bf16_L3000", "bf16_r32_L4096"])
def test_t2_t3_gaussian_inputs(which):
    if which == "config0":
        cfg = wl.get_config(0); ks = wl.k_per_head(cfg).tolist()
    elif which == "bf16_L3000":
        cfg = make_cfg(3000, 128, 16, 3, "bf16", basis_rank=64, scale_num=2.0); ks = [187, 1500, 40]
    else:
        cfg = make_cfg(4096, 128, 32, 2, "bf16", basis_rank=64, scale_num=2.0); ks = [256, 1024]
    case = Case(cfg, ks, names=("Q", "K"))
    p = case.problem(dsv)
    idx = _run_topk(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    Qlr, Klr = dsv.lowrank_project(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    L = cfg.L
    rows = np.unique(np.concatenate([np.arange(0, L, max(L // 61, 1)), [L - 1, L - 2, 31, 32, 33]])).astype(np.int32)
    identical = total = 0
    for h in range(cfg.H):
        got = case.idx_rows(idx, h)
        assert np.all(np.diff(got, axis=1) > 0) and got.min() >= 0 and got.max() < L      # ascending, distinct, in range
        S_gpu = dsv.lowrank_scores_rows(p, Qlr, Klr, 0, h, torch.from_numpy(rows).cuda())
        torch.cuda.synchronize()
        S_gpu = S_gpu.cpu().numpy()
        # the device scores themselves against the oracle's exact scores of the device's projections
        S_ref = oracle.scores(Qlr[0, h, rows].float().cpu().numpy(), Klr[0, h].float().cpu().numpy())
        bound = cfg.r * 2.0 ** -23 * (np.abs(Qlr[0, h, rows].float().cpu().numpy()).astype(np.float64)
                                      @ np.abs(Klr[0, h].float().cpu().numpy()).astype(np.float64).T) + 1e-30
        assert np.all(np.abs(S_gpu - S_ref) <= bound)
        # T2: oracle selection on the device's score bits == device index rows
        assert np.array_equal(oracle.topk_from_scores(S_gpu.astype(np.float64), ks[h]), got[rows]), f"T2 head {h}"
        # T3: against the pure oracle.  Every key on which a row differs must sit inside the rounding band of
        # the oracle's threshold: |S_or[j] - tau_or| <= max_j' e[j'] + e[j], e = fp32 accumulation bound of the
        # r products + the exact effect of projected terms rounded the other way (gpu_util.score_error_bound).
        Qd = Qlr[0, h, rows].float().cpu().numpy()
        Kd = Klr[0, h].float().cpu().numpy()
        idx_ref, Qo, Ko, S_or = oracle.lowrank_topk(case.host["Q"][h][rows], case.host["K"][h], case.Wq[h], case.Wk[h],
                                                    ks[h], cfg.dtype, return_intermediates=True)
        # (Qd, Kd are within one storage ulp of Qo, Ko: test_project_matches_oracle; the bound below uses the
        # exact score difference they cause, so it needs no assumption about them)
        e = score_error_bound(Qd, Kd, S_ref, S_or, cfg.r)
        for a, i in enumerate(rows):
            total += 1
            identical += assert_t3_valid(f"{which} head {h} row {i}", got[i], idx_ref[a], S_or[a], e[a], ks[h])
    print(f"{which}: {identical}/{total} sampled rows identical to the pure fp64 oracle", flush=True)
    # projections can differ by one rounding, scores by fp32 accumulation: most rows still agree exactly
    assert identical / total > 0.5, (identical, total)


def test_k_equals_L_and_k_equals_1():
    cfg = make_cfg(200, 64, 16, 2, "f32")
    case = Case(cfg, [200, 1], names=("Q", "K"))
    p = case.problem(dsv)
    idx = _run_topk(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    assert np.array_equal(case.idx_rows(idx, 0), np.tile(np.arange(200, dtype=np.int32), (200, 1)))
    Qlr, Klr = dsv.lowrank_project(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    S = dsv.lowrank_scores_rows(p, Qlr, Klr, 0, 1, torch.arange(200, dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(case.idx_rows(idx, 1)[:, 0], S.cpu().numpy().argmax(axis=1))


# ------------------------------------------------------------------------------ transposed index
def test_idx_transpose_is_stable_for_any_order_inside_the_rows():
    """dsv_idx_transpose: every list ascending in the query index and identical from run to run, also when the rows
    themselves are in no particular order (the dkdv step of dsv_sparse_attn_bwd relies on it); several query chunks
    per head (L > 64 * 256 would be needed for chunks above the minimum of 64 rows: L = 1500 gives 24 chunks)."""
    L, ks = 1500, [37, 700]
    rng = np.random.default_rng(5)
    rows = [np.stack([rng.permutation(L)[:k] for _ in range(L)]).astype(np.int32) for k in ks]      # unsorted rows
    p = dsv.Problem(1, len(ks), L, 64, 16, "bf16", ks, 1.0)
    flat = torch.from_numpy(np.concatenate([r.reshape(-1) for r in rows])).cuda()
    idx_t, col = dsv.idx_transpose(p, flat)
    idx_t_again, col_again = dsv.idx_transpose(p, flat)
    torch.cuda.synchronize()
    assert torch.equal(idx_t, idx_t_again) and torch.equal(col, col_again)
    idx_t, col = idx_t.cpu().numpy(), col.cpu().numpy()
    off = wl.idx_offsets(1, len(ks), L, ks)
    for h in range(len(ks)):
        _check_transpose(rows[h], idx_t[off[h]:off[h + 1]], col[h], L, sorted_lists=True)


def _check_transpose(idx_rows, idx_t_head, col, L, sorted_lists):
    """idx_rows [L, k]; idx_t_head: the head's block of the key-major index; col [L+1]."""
    k = idx_rows.shape[1]
    counts = np.bincount(idx_rows.reshape(-1), minlength=L)
    assert col[0] == 0 and col[-1] == L * k and np.array_equal(np.diff(col), counts)
    # reference transpose: stable sort of the (query, key) pairs by key keeps queries ascending
    q_of_pair = np.repeat(np.arange(L, dtype=np.int32), k)
    order = np.argsort(idx_rows.reshape(-1), kind="stable")
    ref = q_of_pair[order]
    if sorted_lists:
        assert np.array_equal(idx_t_head, ref)
    else:
        got = idx_t_head.copy()
        for j in range(L):
            got[col[j]:col[j + 1]].sort()
        assert np.array_equal(got, ref)


@pytest.mark.parametrize("kind,dtype,L,d,r,ks", [("ternary", "bf16", 777, 128, 16, [100, 33]),
                                                 ("gauss", "bf16", 3000, 128, 16, [187, 1500, 40]),
                                                 ("gauss", "f32", 1024, 64, 16, [128, 1024]),
                                                 ("ternary", "bf16", 95, 64, 32, [95, 1, 17])])
def test_lowrank_topk_t_emits_the_exact_transpose(kind, dtype, L, d, r, ks):
    H = len(ks)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    if kind == "ternary":
        Qs, Ks, Wqs, Wks = zip(*(wl.ternary_head_tensors(L, d, r, seed=2, head=h) for h in range(H)))
        dev = lambda a: torch.from_numpy(np.stack(a)).cuda().to(td).contiguous()
        Q, K, Wq, Wk = dev(Qs)[None], dev(Ks)[None], dev(Wqs), dev(Wks)
        p = dsv.Problem(1, H, L, d, r, dtype, ks, 1.0)
    else:
        case = Case(make_cfg(L, d, r, H, dtype, basis_rank=32), ks, names=("Q", "K"))
        Q, K, Wq, Wk = case.dev["Q"], case.dev["K"], case.dWq, case.dWk
        p = case.problem(dsv)
    idx_plain = _run_topk(p, Q, K, Wq, Wk)
    idx, idx_t, col = dsv.lowrank_topk_t(p, Q, K, Wq, Wk)
    idx_t2, col2 = dsv.idx_transpose(p, idx)
    torch.cuda.synchronize()
    idx, idx_t, col, idx_t2, col2 = (x.cpu().numpy() for x in (idx, idx_t, col, idx_t2, col2))
    assert np.array_equal(idx, idx_plain)                          # same selection with or without the transpose
    off = wl.idx_offsets(1, H, L, ks)
    for h in range(H):
        rows = idx[off[h]:off[h + 1]].reshape(L, ks[h])
        _check_transpose(rows, idx_t[off[h]:off[h + 1]], col[h], L, sorted_lists=True)
        _check_transpose(rows, idx_t2[off[h]:off[h + 1]], col2[h], L, sorted_lists=True)   # dsv_idx_transpose is stable


# ------------------------------------------------------------------------------ windowed threshold search
@pytest.fixture
def search_mode():
    """Switch the threshold search and put the automatic choice back afterwards."""
    yield dsv.threshold_search
    dsv.threshold_search(0)


def _both_searches(p, Q, K, Wq, Wk):
    dsv.threshold_search(1)
    radix = _run_topk(p, Q, K, Wq, Wk)
    dsv.threshold_search(2)
    window = _run_topk(p, Q, K, Wq, Wk)
    return radix, window


@pytest.mark.parametrize("dtype,L,d,r,ks", [("bf16", 16384, 128, 16, [1024, 64, 4096]), ("bf16", 5000, 64, 32, [313, 2500, 1]),
                                            ("f32", 4100, 64, 16, [4100, 4099, 256]), ("bf16", 8192, 128, 64, [512, 7])])
def test_windowed_search_gives_the_radix_search_result(search_mode, dtype, L, d, r, ks):
    """Gaussian inputs: every row of the index identical under both searches (dense, sparse, k = 1, k = L, k = L - 1,
    ragged last key tile), and sampled rows equal to the oracle's selection on the device's own score bits."""
    case = Case(make_cfg(L, d, r, len(ks), dtype, basis_rank=32, scale_num=2.0), ks, names=("Q", "K"))
    p = case.problem(dsv)
    radix, window = _both_searches(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    assert np.array_equal(radix, window)
    Qlr, Klr = dsv.lowrank_project(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    rows = np.unique(np.concatenate([np.arange(0, L, L // 23), [L - 1, 31, 32]])).astype(np.int32)
    for h in range(len(ks)):
        S_gpu = dsv.lowrank_scores_rows(p, Qlr, Klr, 0, h, torch.from_numpy(rows).cuda())
        torch.cuda.synchronize()
        ref = oracle.topk_from_scores(S_gpu.cpu().numpy().astype(np.float64), ks[h])
        assert np.array_equal(ref, case.idx_rows(window, h)[rows]), f"head {h}"


def test_windowed_search_hands_ties_and_bad_samples_to_the_radix_search(search_mode):
    """Inputs the windowed search cannot settle by itself: scores with massive ties (ternary inputs: bins overflow),
    all scores equal, and keys whose sampled rows say nothing about the rest (the bracket misses the threshold)."""
    L, d, r, ks = 4096, 64, 16, [300, 77]
    H = len(ks)
    Qs, Ks, Wqs, Wks = zip(*(wl.ternary_head_tensors(L, d, r, seed=3, head=h) for h in range(H)))
    dev = lambda a: torch.from_numpy(np.stack(a)).cuda().to(torch.bfloat16).contiguous()
    p = dsv.Problem(1, H, L, d, r, "bf16", ks, 1.0)
    dsv.threshold_search(2)
    idx = _run_topk(p, dev(Qs)[None], dev(Ks)[None], dev(Wqs), dev(Wks))
    off = wl.idx_offsets(1, H, L, ks)
    for h in range(H):
        ref = oracle.lowrank_topk(Qs[h], Ks[h], Wqs[h], Wks[h], ks[h], "bf16")
        assert np.array_equal(idx[off[h]:off[h + 1]].reshape(L, ks[h]), ref), f"ternary head {h}"

    case = Case(make_cfg(L, d, r, 1, "bf16"), [37], names=("Q", "K"))
    p1 = case.problem(dsv)
    idx = _run_topk(p1, torch.zeros_like(case.dev["Q"]), case.dev["K"], case.dWq, case.dWk)
    assert np.array_equal(idx.reshape(L, 37), np.tile(np.arange(37, dtype=np.int32), (L, 1)))

    # the sample takes key rows i * stride + stride / 2 (stride = L / 2048): shrink exactly those rows
    case = Case(make_cfg(L, d, r, 2, "bf16", basis_rank=32, scale_num=2.0), [256, 1000], names=("Q", "K"))
    p2 = case.problem(dsv)
    K = case.dev["K"].clone()
    stride = L // 2048
    K[:, :, stride // 2::stride, :] *= 1.0 / 64
    radix, window = _both_searches(p2, case.dev["Q"], K, case.dWq, case.dWk)
    assert np.array_equal(radix, window)


def test_windowed_search_with_transposed_and_grouped_emission(search_mode):
    """The transposed index and the query-grouped call (fewer query rows than keys) on top of the windowed search."""
    grid, cube, ks = (4, 32, 32), (2, 2, 2), [256, 100]
    L = grid[0] * grid[1] * grid[2]
    case = Case(make_cfg(L, 128, 16, len(ks), "bf16", basis_rank=32, scale_num=2.0), ks, names=("Q", "K"))
    p = case.problem(dsv)
    grp = dsv.Grouping(grid, cube)
    out = {}
    for mode in (1, 2):
        dsv.threshold_search(mode)
        idx, idx_t, col = dsv.lowrank_topk_t(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
        idx_g, idx_t_g, col_g = dsv.lowrank_topk_grouped(p, grp, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
        torch.cuda.synchronize()
        out[mode] = [x.cpu().numpy() for x in (idx, idx_t, col, idx_g, idx_t_g, col_g)]
    for a, b in zip(out[1], out[2]):
        assert np.array_equal(a, b)


def test_windowed_search_over_more_heads_than_one_launch_table_holds(search_mode):
    """70 heads: the (batch, head) pairs go through the kernels 64 at a time, each table with its own list of
    unsettled tiles; ternary inputs in some heads put tiles on those lists."""
    L, d, r, H = 4096, 64, 16, 70
    ks = [256 if h % 3 else 100 for h in range(H)]
    case = Case(make_cfg(L, d, r, H, "bf16", basis_rank=32, scale_num=2.0), ks, names=("Q", "K"))
    Q, K = case.dev["Q"].clone(), case.dev["K"].clone()
    for h in (5, 64, 69):                      # massive ties in heads of both tables
        tq, tk, _, _ = wl.ternary_head_tensors(L, d, r, seed=4, head=h)
        Q[0, h] = torch.from_numpy(tq).to(Q.dtype)
        K[0, h] = torch.from_numpy(tk).to(K.dtype)
    p = case.problem(dsv)
    radix, window = _both_searches(p, Q, K, case.dWq, case.dWk)
    assert np.array_equal(radix, window)
