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
