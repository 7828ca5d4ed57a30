"""The optional index validator (dsv_idx_validate) on good and deliberately bad index rows.  The bad rows
only ever reach the validator, whose kernels read them with bounds-checked logic and exit normally; the
verdict is a host-visible status."""
import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def _idx(L, ks, ascending=True):
    return np.concatenate([wl.random_subset_idx(L, k, L, seed=3, head=h, ascending=ascending).reshape(-1)
                           for h, k in enumerate(ks)])


@pytest.mark.parametrize("L,ks", [(777, [100, 33]), (4096, [512, 1, 4096])])
def test_validator_accepts_valid_rows_and_names_the_first_bad_one(L, ks):
    H = len(ks)
    off = wl.idx_offsets(1, H, L, ks)
    p_sorted = dsv.Problem(1, H, L, 64, 16, "bf16", ks, 0.1, sorted_index=True)
    p_any = dsv.Problem(1, H, L, 64, 16, "bf16", ks, 0.1, sorted_index=False)
    good = _idx(L, ks)
    ok, rep = dsv.idx_validate(p_sorted, torch.from_numpy(good).cuda())
    assert ok and rep == (0, -1, -1)
    ok, rep = dsv.idx_validate(p_any, torch.from_numpy(good).cuda())
    assert ok and rep == (0, -1, -1)
    # rows in random order: fine without the flag, an error with it
    shuffled = _idx(L, ks, ascending=False)
    ok, _ = dsv.idx_validate(p_any, torch.from_numpy(shuffled).cuda())
    assert ok
    if ks[0] > 1:
        ok, rep = dsv.idx_validate(p_sorted, torch.from_numpy(shuffled).cuda())
        assert not ok and rep[0] > 0

    def expect_bad(mutate, head, row, problems=(p_sorted, p_any)):
        bad = good.copy()
        view = bad[off[head]:off[head + 1]].reshape(L, ks[head])
        mutate(view[row])
        for p in problems:
            ok, rep = dsv.idx_validate(p, torch.from_numpy(bad).cuda())
            assert not ok and rep == (1, head, row), (rep, head, row)

    def out_of_range_high(r): r[-1] = L
    def negative(r): r[0] = -1
    expect_bad(out_of_range_high, 0, 5)
    expect_bad(negative, 1, L - 1)
    if ks[0] >= 2:
        def duplicate(r): r[1] = r[0]
        expect_bad(duplicate, 0, L // 2)
        def swapped(r): r[0], r[1] = r[1], r[0]
        expect_bad(swapped, 0, 17, problems=(p_sorted,))        # still distinct and in range: only the order is wrong
    # several bad rows: counted, and the first one reported
    bad = good.copy()
    v = bad[off[0]:off[1]].reshape(L, ks[0])
    v[3, 0] = L + 7
    v[L - 2, 0] = -5
    bad[off[1] + 0] = L
    ok, rep = dsv.idx_validate(p_any, torch.from_numpy(bad).cuda())
    assert not ok and rep == (3, 0, 3)


def test_stage1_output_passes_the_validator():
    from gpu_util import Case, make_cfg
    cfg = make_cfg(3000, 128, 16, 3, "bf16", basis_rank=64, scale_num=2.0)
    case = Case(cfg, [187, 1500, 40], names=("Q", "K"))
    p = case.problem(dsv, sorted_index=True)
    idx = dsv.lowrank_topk(p, case.dev["Q"], case.dev["K"], case.dWq, case.dWk)
    ok, rep = dsv.idx_validate(p, idx)
    assert ok and rep[0] == 0
