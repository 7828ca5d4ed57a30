"""The calls enqueue kernels only (no allocation, no memset nodes, no host synchronisation), so a caller
can record them into a HIP graph.  Capture the whole path once, replay it several times with eager
work and synchronisations in between, and compare every replay with the eager result."""
import numpy as np
import pytest
import torch

import workloads as wl
from gpu_util import Case, make_cfg

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def test_whole_path_replays_from_a_graph():
    L, d, ks = 1500, 128, [96, 40]
    cfg = make_cfg(L, d, 16, len(ks), "bf16", basis_rank=64, scale_num=2.0)
    case = Case(cfg, ks)
    p = case.problem(dsv, sorted_index=True)
    x = case.dev
    nnz = p.nnz
    dev = x["Q"].device
    out = dict(idx=torch.empty(nnz, dtype=torch.int32, device=dev), idx_t=torch.empty(nnz, dtype=torch.int32, device=dev),
               col=torch.empty((cfg.H, L + 1), dtype=torch.int64, device=dev), O=torch.empty_like(x["Q"]),
               lse=torch.empty((1, cfg.H, L), dtype=torch.float32, device=dev), dQ=torch.empty_like(x["Q"]),
               dK=torch.empty_like(x["Q"]), dV=torch.empty_like(x["Q"]))
    ws1 = torch.empty(dsv.lowrank_topk_t_workspace(p), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(dsv.sparse_attn_fwd_workspace(p), dsv.sparse_attn_bwd_t_workspace(p), 256), dtype=torch.uint8, device=dev)

    def whole_path():
        dsv.lowrank_topk_t(p, x["Q"], x["K"], case.dWq, case.dWk, idx=out["idx"], idx_t=out["idx_t"], col_ptr=out["col"],
                           workspace=ws1)
        dsv.sparse_attn_fwd(p, x["Q"], x["K"], x["V"], out["idx"], O=out["O"], lse=out["lse"], workspace=ws2)
        dsv.sparse_attn_bwd_t(p, x["Q"], x["K"], x["V"], out["idx"], out["idx_t"], out["col"], out["O"], out["lse"], x["dO"],
                              dQ=out["dQ"], dK=out["dK"], dV=out["dV"], workspace=ws2)

    whole_path()
    torch.cuda.synchronize()
    eager = {n: t.clone() for n, t in out.items()}

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        whole_path()                      # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        whole_path()
    for rep in range(3):
        for t in out.values():
            t.zero_()                     # eager work between the replays
        scratch = torch.randn(1 << 16, device=dev).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(float(scratch))
        for n, t in out.items():
            assert torch.equal(t, eager[n]), f"replay {rep}: {n} differs from the eager result"


def _replay_and_compare(run, out, dev):
    run()
    torch.cuda.synchronize()
    eager = {n: t.clone() for n, t in out.items()}
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for rep in range(3):
        for t in out.values():
            t.zero_()
        scratch = torch.randn(1 << 16, device=dev).sum()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.isfinite(float(scratch))
        for n, t in out.items():
            assert torch.equal(t, eager[n]), f"replay {rep}: {n} differs from the eager result"


def test_grouped_path_and_own_transposition_replay_from_a_graph():
    """The query-grouped calls (group kernels, L2-blocked form) and dsv_sparse_attn_bwd with its own stable
    transposition enqueue kernels only as well."""
    grid, cube, ks = (4, 16, 32), (2, 2, 2), [160, 64]
    L = grid[0] * grid[1] * grid[2]
    cfg = make_cfg(L, 128, 16, len(ks), "bf16", basis_rank=64, scale_num=2.0)
    case = Case(cfg, ks)
    p = case.problem(dsv, sorted_index=True)
    grp = dsv.Grouping(grid, cube)
    x = case.dev
    dev = x["Q"].device
    n_g = p.nnz // grp.G
    out = dict(idx_g=torch.empty(n_g, dtype=torch.int32, device=dev), idx_t_g=torch.empty(n_g, dtype=torch.int32, device=dev),
               col=torch.empty((cfg.H, L + 1), dtype=torch.int64, device=dev), O=torch.empty_like(x["Q"]),
               lse=torch.empty((1, cfg.H, L), dtype=torch.float32, device=dev), dQ=torch.empty_like(x["Q"]),
               dK=torch.empty_like(x["Q"]), dV=torch.empty_like(x["Q"]))
    ws1 = torch.empty(dsv.lowrank_topk_grouped_workspace(p, grp), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(dsv.sparse_attn_fwd_grouped_workspace(p, grp), dsv.sparse_attn_bwd_grouped_workspace(p, grp), 256),
                      dtype=torch.uint8, device=dev)

    def grouped_path():
        dsv.lowrank_topk_grouped(p, grp, x["Q"], x["K"], case.dWq, case.dWk, idx_g=out["idx_g"], idx_t_g=out["idx_t_g"],
                                 col_ptr=out["col"], workspace=ws1)
        dsv.sparse_attn_fwd_grouped(p, grp, x["Q"], x["K"], x["V"], out["idx_g"], O=out["O"], lse=out["lse"], workspace=ws2)
        dsv.sparse_attn_bwd_grouped(p, grp, x["Q"], x["K"], x["V"], out["idx_g"], out["idx_t_g"], out["col"], out["O"], out["lse"],
                                    x["dO"], dQ=out["dQ"], dK=out["dK"], dV=out["dV"], workspace=ws2)

    _replay_and_compare(grouped_path, out, dev)

    # per-query path through dsv_sparse_attn_bwd (builds the key-major index itself)
    out2 = dict(idx=torch.empty(p.nnz, dtype=torch.int32, device=dev), O=torch.empty_like(x["Q"]),
                lse=torch.empty((1, cfg.H, L), dtype=torch.float32, device=dev), dQ=torch.empty_like(x["Q"]),
                dK=torch.empty_like(x["Q"]), dV=torch.empty_like(x["Q"]))
    ws3 = torch.empty(dsv.lowrank_topk_workspace(p), dtype=torch.uint8, device=dev)
    ws4 = torch.empty(max(dsv.sparse_attn_fwd_workspace(p), dsv.sparse_attn_bwd_workspace(p), 256), dtype=torch.uint8, device=dev)

    def own_transposition():
        dsv.lowrank_topk(p, x["Q"], x["K"], case.dWq, case.dWk, idx=out2["idx"], workspace=ws3)
        dsv.sparse_attn_fwd(p, x["Q"], x["K"], x["V"], out2["idx"], O=out2["O"], lse=out2["lse"], workspace=ws4)
        dsv.sparse_attn_bwd(p, x["Q"], x["K"], x["V"], out2["idx"], out2["O"], out2["lse"], x["dO"], dQ=out2["dQ"],
                            dK=out2["dK"], dV=out2["dV"], workspace=ws4)

    _replay_and_compare(own_transposition, out2, dev)
