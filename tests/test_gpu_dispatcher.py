"""The memory column of the dispatcher table (bench.py --dispatcher-table): the bytes bench.path_memory reports
are the library's own workspace queries plus the index tensors, and buffers of exactly those sizes carry the
whole path."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import Case, make_cfg

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def test_reported_bytes_are_the_workspace_queries_and_suffice():
    import bench
    cfg = make_cfg(20000, 128, 16, 2, "bf16", basis_rank=64, scale_num=2.0)       # large enough for the L2-blocked kernels
    ks = [1250, 400]
    case = Case(cfg, ks)
    p = case.problem(dsv, sorted_index=True)
    mem = bench.path_memory(dsv, p)
    assert mem["workspace"] == {"lowrank_topk_t": dsv.lowrank_topk_t_workspace(p), "sparse_attn_fwd": dsv.sparse_attn_fwd_workspace(p),
                                "sparse_attn_bwd_dq": dsv.sparse_attn_bwd_dq_workspace(p),
                                "sparse_attn_bwd_dkdv": dsv.sparse_attn_bwd_dkdv_workspace(p)}
    assert mem["workspace"]["sparse_attn_fwd"] > 0                                 # the blocked kernels are in use
    nnz = cfg.L * sum(ks)
    assert mem["tensors"]["idx"] == mem["tensors"]["idx_t"] == 4 * nnz
    assert mem["tensors"]["col_ptr"] == 2 * (cfg.L + 1) * 8
    assert mem["peak_bytes"] == sum(mem["tensors"].values()) + max(mem["workspace"].values())
    # exactly these sizes are enough: every call succeeds with them, one byte less is refused
    dev = "cuda:0"
    buf = lambda n: torch.empty(n, dtype=torch.uint8, device=dev)
    idx, idx_t = (torch.empty(nnz, dtype=torch.int32, device=dev) for _ in range(2))
    col = torch.empty((2, cfg.L + 1), dtype=torch.int64, device=dev)
    d = case.dev
    dsv.lowrank_topk_t(p, d["Q"], d["K"], case.dWq, case.dWk, idx=idx, idx_t=idx_t, col_ptr=col,
                       workspace=buf(mem["workspace"]["lowrank_topk_t"]))
    O, lse = dsv.sparse_attn_fwd(p, d["Q"], d["K"], d["V"], idx, workspace=buf(mem["workspace"]["sparse_attn_fwd"]))
    dQ, delta = dsv.sparse_attn_bwd_dq(p, d["Q"], d["K"], d["V"], idx, O, lse, d["dO"],
                                       workspace=buf(mem["workspace"]["sparse_attn_bwd_dq"]))
    dsv.sparse_attn_bwd_dkdv(p, d["Q"], d["K"], d["V"], idx_t, col, lse, delta, d["dO"],
                             workspace=buf(mem["workspace"]["sparse_attn_bwd_dkdv"]))
    torch.cuda.synchronize()
    with pytest.raises(dsv.DsvError):
        dsv.sparse_attn_fwd(p, d["Q"], d["K"], d["V"], idx, workspace=buf(mem["workspace"]["sparse_attn_fwd"] - 256))


def test_crossover_interpolation():
    import bench
    assert bench.interpolate_crossover([(0.01, 100.0), (0.02, 200.0), (0.04, 400.0)], 300.0) == 0.03
    assert bench.interpolate_crossover([(0.01, 100.0), (0.02, 200.0)], 500.0) is None
    assert bench.interpolate_crossover([(0.01, 100.0), (0.02, 200.0)], 50.0) is None
