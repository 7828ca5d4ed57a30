"""GPU parity of stage 2 (dsv_sparse_attn_fwd / dsv_sparse_attn_bwd) against the CPU oracle, on the
oracle's own index sets, through the C ABI.  Tolerance: max-abs 2e-2 (bf16) / 1e-4 (fp32) against the
fp64 oracle, widened to 2^-7 |ref| (bf16) / 2^-20 |ref| (fp32) where the reference exceeds ~2.5."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from gpu_util import Case, assert_close, make_cfg

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def _oracle_idx(case):
    """Per head: the oracle's top-k rows for the case's inputs (the real selection)."""
    out = []
    for h in range(case.cfg.H):
        out.append(oracle.lowrank_topk(case.host["Q"][h], case.host["K"][h], case.Wq[h], case.Wk[h], case.ks[h],
                                       case.cfg.dtype))
    return out


def _run_stage2(case, idx_rows, sorted_index=False):
    p = case.problem(dsv, sorted_index=sorted_index)
    flat = torch.from_numpy(np.concatenate([r.reshape(-1) for r in idx_rows])).cuda()
    d = case.dev
    O, lse = dsv.sparse_attn_fwd(p, d["Q"], d["K"], d["V"], flat)
    dQ, dK, dV = dsv.sparse_attn_bwd(p, d["Q"], d["K"], d["V"], flat, O, lse, d["dO"])
    torch.cuda.synchronize()
    if sorted_index:
        # the same backward with an ascending transposed index supplied: both steps L2-blocked.
        # The reference transpose is a stable sort of the pairs by key (plain numpy, no library code).
        idx_t, col = [], []
        for h, rows in enumerate(idx_rows):
            L, k = rows.shape
            order = np.argsort(rows.reshape(-1), kind="stable")
            idx_t.append((order // k).astype(np.int32))
            col.append(np.concatenate([[0], np.cumsum(np.bincount(rows.reshape(-1), minlength=L))]).astype(np.int64))
        idx_t = torch.from_numpy(np.concatenate(idx_t)).cuda()
        col = torch.from_numpy(np.stack(col)).cuda()
        dQ2, dK2, dV2 = dsv.sparse_attn_bwd_t(p, d["Q"], d["K"], d["V"], flat, idx_t, col, O, lse, d["dO"])
        torch.cuda.synchronize()
        # dsv_sparse_attn_bwd builds the same (stable) transposed index itself: identical results, bit for bit
        assert torch.equal(dQ2, dQ) and torch.equal(dK2, dK) and torch.equal(dV2, dV)
        return O, lse, dQ2, dK2, dV2
    return O, lse, dQ, dK, dV


def _check_all(case, idx_rows, outs):
    O, lse, dQ, dK, dV = outs
    cfg = case.cfg
    worst = {}
    for h in range(cfg.H):
        Q, K, V, dO = (case.host[n][h] for n in ("Q", "K", "V", "dO"))
        O_ref, lse_ref = oracle.sparse_fwd(Q, K, V, idx_rows[h], cfg.scale)
        dQ_ref, dK_ref, dV_ref = oracle.sparse_bwd(Q, K, V, idx_rows[h], dO, cfg.scale)
        for name, got, ref in (("O", O[0, h], O_ref), ("dQ", dQ[0, h], dQ_ref), ("dK", dK[0, h], dK_ref),
                               ("dV", dV[0, h], dV_ref)):
            worst[name] = max(worst.get(name, 0.0), assert_close(f"{name}[h={h}]", got, ref, cfg.dtype))
        worst["lse"] = max(worst.get("lse", 0.0), assert_close(f"lse[h={h}]", lse[0, h], lse_ref, "f32"))
    return worst


def test_config0_full():
    cfg = wl.get_config(0)
    case = Case(cfg, wl.k_per_head(cfg))
    idx_rows = _oracle_idx(case)
    print(_check_all(case, idx_rows, _run_stage2(case, idx_rows)))


@pytest.mark.parametrize("dtype,L,d,ks", [("bf16", 1000, 128, [64, 250, 7]), ("bf16", 513, 64, [513, 1]),
                                          ("f32", 300, 128, [33, 300]), ("bf16", 2048, 128, [128, 126])])
def test_ragged_sizes_and_mixed_k(dtype, L, d, ks):
    cfg = make_cfg(L, d, 16, len(ks), dtype, basis_rank=64 if d == 128 else 32, scale_num=2.0)
    case = Case(cfg, ks)
    idx_rows = _oracle_idx(case)
    print(_check_all(case, idx_rows, _run_stage2(case, idx_rows)))


@pytest.mark.parametrize("dtype,L,d,ks", [("bf16", 9000, 128, [300, 64]), ("f32", 5000, 128, [40, 700]),
                                          ("bf16", 8200, 64, [1, 8200])])
def test_l2_blocked_kernels_on_sorted_indices(dtype, L, d, ks):
    """Several key ranges with a ragged last one; DSV_FLAG_SORTED_INDEX set."""
    cfg = make_cfg(L, d, 16, len(ks), dtype, basis_rank=64 if d == 128 else 32, scale_num=2.0)
    case = Case(cfg, ks)
    idx_rows = _oracle_idx(case)
    print(_check_all(case, idx_rows, _run_stage2(case, idx_rows, sorted_index=True)))


def test_row_order_does_not_matter_and_unselected_keys_get_zero():
    L, d, k = 640, 128, 48
    cfg = make_cfg(L, d, 16, 1, "bf16", basis_rank=64, scale_num=2.0)
    case = Case(cfg, [k])
    idx = wl.random_subset_idx(L - 40, k, L, seed=5, ascending=False)       # keys >= L-40 never selected, rows shuffled
    outs = _run_stage2(case, [idx])
    _check_all(case, [idx], outs)
    assert torch.all(outs[3][0, 0, L - 40:] == 0) and torch.all(outs[4][0, 0, L - 40:] == 0)


def test_k_equals_L_is_dense_attention():
    L, d = 256, 64
    cfg = make_cfg(L, d, 16, 1, "f32")
    case = Case(cfg, [L])
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    O, lse, dQ, dK, dV = _run_stage2(case, [idx])
    Q, K, V, dO = (case.host[n][0] for n in ("Q", "K", "V", "dO"))
    O_ref, lse_ref = oracle.dense_fwd(Q, K, V, cfg.scale)
    dQ_ref, dK_ref, dV_ref = oracle.dense_bwd(Q, K, V, dO, cfg.scale)
    for name, got, ref in (("O", O, O_ref), ("lse", lse, lse_ref), ("dQ", dQ, dQ_ref), ("dK", dK, dK_ref), ("dV", dV, dV_ref)):
        assert_close(name, got[0, 0], ref, "f32")


def test_kernel_timing_spans():
    """The measurement aid: spans report a positive time after a call, results are unchanged, and a
    span that has not run since timing was switched on is an error."""
    L, d, k = 640, 128, 48
    cfg = make_cfg(L, d, 16, 1, "bf16", basis_rank=64, scale_num=2.0)
    case = Case(cfg, [k])
    idx = wl.random_subset_idx(L, k, L, seed=6, ascending=True)
    plain = _run_stage2(case, [idx], sorted_index=True)
    dsv.kernel_timing(True)
    try:
        with pytest.raises(dsv.DsvError):
            dsv.kernel_ms("fwd_sweep")
        timed = _run_stage2(case, [idx], sorted_index=True)
        for span in ("fwd_sweep", "dq_sweep", "dkdv_sweep"):
            ms = dsv.kernel_ms(span)
            assert 0.0 < ms < 1000.0, (span, ms)
        with pytest.raises(dsv.DsvError):
            dsv.kernel_ms("emit")
    finally:
        dsv.kernel_timing(False)
    for a, b in zip(plain, timed):
        assert torch.equal(a, b)
