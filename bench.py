#!/usr/bin/env python3
"""Benchmark of the DSV sparse-attention hot path on one MI355X.

One step = one pass of the whole path over one synthetic batch that is already resident in HBM:
    stage 1  dsv_lowrank_topk_t        (project, threshold search, emit idx and its transpose)
    stage 2  dsv_sparse_attn_fwd
             dsv_sparse_attn_bwd_dq, dsv_sparse_attn_bwd_dkdv
             (the two steps dsv_sparse_attn_bwd_t runs, called one by one so that each can be timed)
Workload: the L = 128k configuration of the benchmark list (6 heads = one GPU's head-parallel share
of 24, d = 128, r = 16, k = 8192 per query, bf16).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--no-dense] [--no-cpu-baseline]
                    [--density-sweep] [--unsorted] [--calibration-copy-mib N]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0       # MI355X HBM3E, published
VALU_LANE_OPS_PER_S = 256 * 64 * 2.4e9   # 256 CUs x 64 fp32 lanes x 2.4 GHz, one (unpacked) VALU op per lane per clock

# HBM traffic of the stage-2 sweeps at config 2, bytes per launch, from two rocprofv3 --pmc runs (FETCH_SIZE,
# WRITE_SIZE, in KiB), each scaled by what the same counter reads for a plain 1 GiB elementwise copy in the same run
# (FETCH_SIZE reads 0.5 GiB for it: factor 2.0; WRITE_SIZE reads 1 GiB: factor 1.0), and the L2 hit rate from
# TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum).  Source: profiles/config2_pmc_counters.md.  The figures belong to ONE
# build of the kernels: they are reported only while the library still names that version.
PMC_LIBRARY_VERSION = "dsv 0.4 (gfx950)"
PMC_CONFIG2 = {
    "sparse_attn_fwd": {"fetch_kib": 31042322, "write_kib": 14155844, "l2_hit_rate": 0.9693},
    "sparse_attn_bwd_dq": {"fetch_kib": 48468979, "write_kib": 12976401, "l2_hit_rate": 0.9644},
    "sparse_attn_bwd_dkdv": {"fetch_kib": 33568648, "write_kib": 12582918, "l2_hit_rate": 0.9739},
}
# the gather sweep inside each stage-2 call (the kernel the roofline object is about)
SWEEP_OF_CALL = {"sparse_attn_fwd": "fwd_sweep", "sparse_attn_bwd_dq": "dq_sweep", "sparse_attn_bwd_dkdv": "dkdv_sweep"}
# Vector memory path (L2 -> vector L1 -> registers): 64 bytes per clock per CU, 256 CUs, 2.4 GHz.  The sweeps'
# gathers are served by it (L2 hit rate 96-98 %); it is what bounds them.
L1_PEAK_GBS = 256 * 64 * 2.4
# What a kernel that ONLY gathers (same lane layout, index staging and block order, no arithmetic) reaches on this
# path: bench.py --gather-ceiling, summary in profiles/gather_ceiling.md (index streamed from memory, 4 MB ranges).
GATHER_CEILING_GBS = {"sparse_attn_fwd": 34241.5, "sparse_attn_bwd_dq": 33888.4, "sparse_attn_bwd_dkdv": 33888.4}
MFMA_BF16_PEAK_TFLOPS = 2500.0


def pmc_traffic_bytes(call):
    c = PMC_CONFIG2[call]
    return int((c["fetch_kib"] * 2.0 + c["write_kib"] * 1.0) * 1024)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=2, help="index into the benchmark config list (headline: 2)")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--unsorted", action="store_true", help="do not set DSV_FLAG_SORTED_INDEX (plain gather kernels)")
    ap.add_argument("--no-dense", action="store_true", help="skip the dense-attention comparator")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip timing the CPU oracle")
    ap.add_argument("--cpu-rows", type=int, default=0, help="query rows of the oracle sample (0 = auto)")
    ap.add_argument("--density-sweep", action="store_true",
                    help="also time the whole path at k/L = 0.5 .. 12.5 %% (same shape) and report the crossover with dense")
    ap.add_argument("--gather-ceiling", action="store_true",
                    help="instead of the benchmark line: run the library's pure-gather probe (dsv_measure_gather_ceiling) and print "
                         "the rate the vector memory path sustains for the stage-2 access pattern")
    ap.add_argument("--dispatcher-table", action="store_true",
                    help="instead of the benchmark line: the offline table a sparse/dense dispatcher consumes -- for L in "
                         "{32k, 64k, 128k} and k/L from 0.5 to 12.5 %%, ms per stage, speedup over dense, and the bytes of "
                         "index and workspace the sparse path needs")
    ap.add_argument("--predictor", action="store_true",
                    help="(default for bf16, d = 128 configs) also time the predictor side at the same shape: approximation "
                         "loss + gradients and the sparsity profiler, both on L/16 sampled query rows")
    ap.add_argument("--no-predictor", action="store_true", help="skip the predictor-side timings")
    ap.add_argument("--grouped", action="store_true",
                    help="(default for bf16, d = 128 configs) also time the query-grouped variant (2 x 2 x 2 cubes) at the "
                         "same shape, and measure what the shared rows cost in accuracy on spatially smooth inputs")
    ap.add_argument("--no-grouped", action="store_true", help="skip the query-grouped variant")
    ap.add_argument("--grouped-cubes", action="store_true",
                    help="with the grouped report: the grouped step also for 2 x 2 x 4 and 2 x 4 x 4 cubes (16 and 32 queries per group)")
    ap.add_argument("--grouped-density-sweep", action="store_true",
                    help="with --grouped: the grouped step at k/L = 3.1 ... 25 % and its interpolated crossover with dense")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="before the steps, run one plain elementwise copy kernel (x + 0 over this many MiB of int32) "
                         "so that a rocprofv3 --pmc run holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    return ap.parse_args()


def upload_inputs(cfg, seed, dev, torch, wl):
    td = torch.bfloat16 if cfg.dtype == "bf16" else torch.float32
    shape = (1, cfg.H, cfg.L, cfg.d)
    g = {n: torch.empty(shape, dtype=td, device=dev) for n in ("Q", "K", "V", "dO")}
    Wq = torch.empty((cfg.H, cfg.d, cfg.r), dtype=td, device=dev)
    Wk = torch.empty((cfg.H, cfg.d, cfg.r), dtype=td, device=dev)
    for h in range(cfg.H):
        t = wl.head_tensors(cfg, h, seed=seed)
        for n in g:
            g[n][0, h].copy_(torch.from_numpy(t[n]).to(td))
        wq, wk = wl.predictor_weights(cfg, h, seed=seed)
        Wq[h].copy_(torch.from_numpy(wq).to(td))
        Wk[h].copy_(torch.from_numpy(wk).to(td))
    return g, Wq, Wk


class Path:
    """Device buffers of one problem, allocated once, and the step that runs the whole path."""
    NAMES = ("lowrank_topk_t", "sparse_attn_fwd", "sparse_attn_bwd_dq", "sparse_attn_bwd_dkdv")

    def __init__(self, dsv, torch, cfg, ks, g, Wq, Wk, sorted_index):
        self.dsv, self.torch, self.g, self.Wq, self.Wk = dsv, torch, g, Wq, Wk
        dev = g["Q"].device
        # stage 1 writes ascending rows and lists, so stage 2 may be told so (DSV_FLAG_SORTED_INDEX)
        self.p = p = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, [int(k) for k in ks], cfg.scale,
                                 sorted_index=sorted_index)
        self.nnz = p.nnz
        self.idx = torch.empty(p.nnz, dtype=torch.int32, device=dev)
        self.idx_t = torch.empty(p.nnz, dtype=torch.int32, device=dev)
        self.col_ptr = torch.empty((cfg.H, cfg.L + 1), dtype=torch.int64, device=dev)
        self.O, self.dQ, self.dK, self.dV = (torch.empty_like(g["Q"]) for _ in range(4))
        self.lse = torch.empty((1, cfg.H, cfg.L), dtype=torch.float32, device=dev)
        self.delta = torch.empty((1, cfg.H, cfg.L), dtype=torch.float32, device=dev)
        self.ws1 = torch.empty(dsv.lowrank_topk_t_workspace(p), dtype=torch.uint8, device=dev)
        self.ws2 = torch.empty(max(dsv.sparse_attn_fwd_workspace(p), dsv.sparse_attn_bwd_dq_workspace(p),
                                   dsv.sparse_attn_bwd_dkdv_workspace(p), 256), dtype=torch.uint8, device=dev)

    def calls(self):
        d, p, g = self.dsv, self.p, self.g
        return (
            lambda: d.lowrank_topk_t(p, g["Q"], g["K"], self.Wq, self.Wk, idx=self.idx, idx_t=self.idx_t,
                                     col_ptr=self.col_ptr, workspace=self.ws1),
            lambda: d.sparse_attn_fwd(p, g["Q"], g["K"], g["V"], self.idx, O=self.O, lse=self.lse, workspace=self.ws2),
            lambda: d.sparse_attn_bwd_dq(p, g["Q"], g["K"], g["V"], self.idx, self.O, self.lse, g["dO"], dQ=self.dQ,
                                         delta=self.delta, workspace=self.ws2),
            lambda: d.sparse_attn_bwd_dkdv(p, g["Q"], g["K"], g["V"], self.idx_t, self.col_ptr, self.lse, self.delta,
                                           g["dO"], dK=self.dK, dV=self.dV, workspace=self.ws2),
        )

    def time(self, steps, warmup):
        """(ms_per_step by the host clock around `steps` steps, per-call ms from events on the launch stream,
        per-kernel ms from the library's own events around single kernels, same stream, averaged over the steps)."""
        torch = self.torch
        spans = self.dsv.KERNEL_SPANS
        kern_ms = {s: 0.0 for s in spans}
        calls = self.calls()
        for _ in range(warmup):
            for c in calls:
                c()
        torch.cuda.synchronize()
        events = []
        self.dsv.kernel_timing(True)
        t0 = time.perf_counter()
        for step in range(steps):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)]
            ev[0].record()
            for i, c in enumerate(calls):
                c()
                ev[i + 1].record()
            events.append(ev)
            # the library keeps one event pair per kernel, so they are read once per step; the read waits for
            # this step's kernels (the wait is inside the timed region: ms_per_step includes it)
            for s in spans:
                kern_ms[s] += self.dsv.kernel_ms(s) / steps
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        self.dsv.kernel_timing(False)
        call_ms = {n: sum(ev[i].elapsed_time(ev[i + 1]) for ev in events) / steps for i, n in enumerate(self.NAMES)}
        return wall_ms, call_ms, kern_ms


def path_memory(dsv, p):
    """Bytes of device memory the sparse path needs beyond Q, K, V, O and the gradients, for problem p (sorted-index
    flag as set in p): both index tensors, the column pointers, lse and Delta, and each call's workspace as the
    library's own queries report it.  Stage 2's workspaces are never live together (one buffer of the largest size)."""
    nbh = p.B * p.H
    ws = {"lowrank_topk_t": dsv.lowrank_topk_t_workspace(p), "sparse_attn_fwd": dsv.sparse_attn_fwd_workspace(p),
          "sparse_attn_bwd_dq": dsv.sparse_attn_bwd_dq_workspace(p), "sparse_attn_bwd_dkdv": dsv.sparse_attn_bwd_dkdv_workspace(p)}
    fixed = {"idx": p.nnz * 4, "idx_t": p.nnz * 4, "col_ptr": nbh * (p.L + 1) * 8, "lse": nbh * p.L * 4, "delta": nbh * p.L * 4}
    peak = sum(fixed.values()) + max(ws["lowrank_topk_t"], max(ws["sparse_attn_fwd"], ws["sparse_attn_bwd_dq"], ws["sparse_attn_bwd_dkdv"]))
    return {"tensors": fixed, "workspace": ws, "peak_bytes": int(peak)}


def dispatcher_table(dsv, torch, np, wl, args):
    """Sec. "Two-Stage DiT Training" (stage 2): the dispatcher enables sparse attention for a block when the
    measured speedup at the block's sparsity and token length pays and the index memory fits; this is that offline
    measurement on this GPU."""
    dev = torch.device("cuda:0")
    import torch.nn.functional as F
    rows = []
    for ci in (1, 3, 2):                       # L = 32k (24 heads), 64k (24 heads), 128k (6 heads)
        cfg = wl.get_config(ci)
        g, Wq, Wk = upload_inputs(cfg, args.seed, dev, torch, wl)
        q = g["Q"].clone().requires_grad_(True); k_ = g["K"].clone().requires_grad_(True); v = g["V"].clone().requires_grad_(True)
        def dense():
            o = F.scaled_dot_product_attention(q, k_, v, scale=cfg.scale)
            o.backward(g["dO"])
            q.grad = k_.grad = v.grad = None
        dense_ms = _time_calls(torch, (dense,), 2, 2)[0]
        del q, k_, v
        torch.cuda.empty_cache()
        for frac in (0.005, 0.01, 0.02, 0.03125, 0.0625, 0.10, 0.125):
            kk = max(1, int(round(cfg.L * frac)))
            pth = Path(dsv, torch, cfg, [kk] * cfg.H, g, Wq, Wk, sorted_index=True)
            ms = _time_calls(torch, pth.calls(), 2, 1)
            mem = path_memory(dsv, pth.p)
            total = sum(ms)
            rows.append({"L": cfg.L, "H": cfg.H, "r": cfg.r, "density": frac, "k": kk,
                         "stage1_ms": round(ms[0], 2), "fwd_ms": round(ms[1], 2), "bwd_ms": round(ms[2] + ms[3], 2),
                         "total_ms": round(total, 2), "dense_ms": round(dense_ms, 2),
                         "speedup_over_dense": round(dense_ms / total, 3),
                         "index_bytes": mem["tensors"]["idx"] + mem["tensors"]["idx_t"],
                         "workspace_bytes": max(mem["workspace"].values()), "peak_extra_bytes": mem["peak_bytes"]})
            print(json.dumps(rows[-1]), file=sys.stderr, flush=True)
            del pth
            torch.cuda.empty_cache()
        del g, Wq, Wk
        torch.cuda.empty_cache()
    # crossover density per L: linear interpolation of total_ms between the swept densities around dense_ms
    cross = {}
    for L in sorted({r["L"] for r in rows}):
        rr = sorted((r for r in rows if r["L"] == L), key=lambda r: r["density"])
        cross[str(L)] = interpolate_crossover([(r["density"], r["total_ms"]) for r in rr], rr[0]["dense_ms"])
    return {"table": rows, "crossover_density": cross,
            "note": "sparse path = lowrank_topk_t + sparse_attn_fwd + sparse_attn_bwd_dq + sparse_attn_bwd_dkdv (sorted-index "
                    "kernels), bf16, d = 128; dense = torch scaled_dot_product_attention fwd+bwd on the same GPU"}


def gather_ceiling(dsv, torch):
    """Rates of the pure-gather probe for the two range sizes the sweeps use (2 MB of K+V rows: forward; 4 MB:
    backward), with the index streamed from memory (one index row per query, as in the real sweeps) and with a
    cached index (64 shared rows).  Same selected fraction as config 2 (1/16 of a range's rows per query)."""
    dev = torch.device("cuda:0")
    L, nq = 131072, 32768
    K = torch.randn((L, 128), device=dev).to(torch.bfloat16)
    V = torch.randn((L, 128), device=dev).to(torch.bfloat16)
    res = []
    for range_rows in (4096, 8192):
        n_ranges, k = L // range_rows, range_rows // 16
        step = range_rows // k
        for idx_rows in (nq, 64):
            g = torch.Generator(device=dev).manual_seed(0)
            idx = (torch.arange(k, device=dev, dtype=torch.int32)[None, None, :] * step +
                   torch.randint(0, step, (n_ranges, idx_rows, k), device=dev, dtype=torch.int32, generator=g)).contiguous()
            out = torch.empty((n_ranges, nq), dtype=torch.int32, device=dev)
            ms = dsv.measure_gather_ceiling(n_ranges, range_rows, nq, k, idx_rows, K, V, idx, out, reps=5)
            nbytes = n_ranges * nq * k * 512
            res.append({"range_bytes": range_rows * 512, "index": "streamed" if idx_rows == nq else "cached (64 rows)",
                        "ms": round(ms, 3), "gathered_bytes": nbytes, "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1),
                        "bytes_per_clk_per_cu": round(nbytes / (ms * 1e-3) / (256 * 2.4e9), 2),
                        "frac_of_path_peak": round(nbytes / (ms * 1e-3) / 1e9 / L1_PEAK_GBS, 4)})
            del idx, out
    return {"probe": "dsv_measure_gather_ceiling: 4 lanes per row, 4 keys per step, K row + V row (2 x 256 B) per index entry, "
                     "no arithmetic; L = 131072 rows, 32768 queries per range",
            "path_peak_GBps": round(L1_PEAK_GBS, 1), "results": res}


def interpolate_crossover(points, dense_ms):
    """points: (density, ms) ascending in density.  Density at which the sparse path takes as long as dense
    (linear between the two swept densities that bracket it); None if it never does inside the sweep."""
    for (d0, m0), (d1, m1) in zip(points, points[1:]):
        if m0 <= dense_ms < m1:
            return round(d0 + (d1 - d0) * (dense_ms - m0) / (m1 - m0), 4)
    return None


def _time_calls(torch, calls, steps, warmup):
    for _ in range(warmup):
        for c in calls:
            c()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(calls) + 1)] for _ in range(steps)]
    for s in range(steps):
        ev[s][0].record()
        for i, c in enumerate(calls):
            c()
            ev[s][i + 1].record()
    torch.cuda.synchronize()
    return [sum(e[i].elapsed_time(e[i + 1]) for e in ev) / steps for i in range(len(calls))]


def grouped_report(dsv, torch, np, wl, cfg, ks, g, Wq, Wk, steps, warmup, dense_ms, per_query_ms, cube=(2, 2, 2)):
    """The query-grouped variant at the same shape (2 x 2 x 2 cubes of the latent grid): one step =
    dsv_lowrank_topk_grouped + dsv_sparse_attn_fwd_grouped + dsv_sparse_attn_bwd_grouped."""
    grp = dsv.Grouping(cfg.grid, cube)
    # stage 1 writes ascending rows and lists: the L2-blocked kernels may be used
    p = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, [int(k) for k in ks], cfg.scale, sorted_index=True)
    dev = g["Q"].device
    n = p.nnz // grp.G
    idx_g = torch.empty(n, dtype=torch.int32, device=dev)
    idx_t_g = torch.empty(n, dtype=torch.int32, device=dev)
    col = torch.empty((cfg.H, cfg.L + 1), dtype=torch.int64, device=dev)
    O, dQ, dK, dV = (torch.empty_like(g["Q"]) for _ in range(4))
    lse = torch.empty((1, cfg.H, cfg.L), dtype=torch.float32, device=dev)
    ws1 = torch.empty(dsv.lowrank_topk_grouped_workspace(p, grp), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(dsv.sparse_attn_bwd_grouped_workspace(p, grp), dsv.sparse_attn_fwd_grouped_workspace(p, grp)),
                      dtype=torch.uint8, device=dev)
    calls = (
        lambda: dsv.lowrank_topk_grouped(p, grp, g["Q"], g["K"], Wq, Wk, idx_g=idx_g, idx_t_g=idx_t_g, col_ptr=col, workspace=ws1),
        lambda: dsv.sparse_attn_fwd_grouped(p, grp, g["Q"], g["K"], g["V"], idx_g, O=O, lse=lse, workspace=ws2),
        lambda: dsv.sparse_attn_bwd_grouped(p, grp, g["Q"], g["K"], g["V"], idx_g, idx_t_g, col, O, lse, g["dO"], dQ=dQ, dK=dK,
                                            dV=dV, workspace=ws2),
    )
    ms = _time_calls(torch, calls, steps, warmup)
    dsv.kernel_timing(True)
    for c in calls:
        c()
    kern = {s_: round(dsv.kernel_ms(s_), 3) for s_ in ("fwd_sweep", "dq_sweep", "dkdv_sweep")}
    dsv.kernel_timing(False)
    total = sum(ms)
    nnz = p.nnz
    out = {"cube": list(cube), "G": grp.G, "ms_per_step": round(total, 3), "kernel_ms": kern,
           "stage_ms": {"lowrank_topk_grouped": round(ms[0], 3), "sparse_attn_fwd_grouped": round(ms[1], 3),
                        "sparse_attn_bwd_grouped": round(ms[2], 3)},
           "speedup_over_dense": round(dense_ms / total, 3) if dense_ms else None,
           "speedup_over_per_query_path": round(per_query_ms / total, 3),
           "index_bytes": {"idx_g": int(n) * 4, "per_query_idx": int(nnz) * 4,
                           "bwd_workspace": int(ws2.numel())},
           # forward: each K / V row crosses the vector memory path once per GROUP
           "fwd_gather_bytes_per_pair": round((2 * cfg.d * 2 + 4) / grp.G, 1),
           "fwd_pairs_per_s": round(nnz / (ms[1] * 1e-3), 1)}
    del ws1, ws2, idx_g, idx_t_g, col, O, dQ, dK, dV, lse
    torch.cuda.empty_cache()
    return out


def predictor_report(dsv, torch, cfg, ks, g, Wq, Wk):
    """dsv_predictor_loss and dsv_profile_sparsity at the benchmark shape, on every 16th query row (the sampling
    factor the paper names)."""
    dev = g["Q"].device
    p = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, [int(k) for k in ks], cfg.scale)
    rows = torch.arange(0, cfg.L, 16, dtype=torch.int32, device=dev)
    n = int(rows.numel())
    ws1 = torch.empty(dsv.predictor_loss_workspace(p, n), dtype=torch.uint8, device=dev)
    ws2 = torch.empty(max(int(dsv.load_library().dsv_profile_sparsity_workspace(p.c, n)), 256), dtype=torch.uint8, device=dev)
    ema = torch.full((cfg.H,), 0.9, dtype=torch.float32, device=dev)
    res = {}
    calls = (lambda: res.__setitem__("loss", dsv.predictor_loss(p, g["Q"], g["K"], Wq, Wk, rows, workspace=ws1)),
             lambda: res.__setitem__("prof", dsv.profile_sparsity(p, g["Q"], g["K"], rows, mass=0.9, ema=ema, alpha=0.1, workspace=ws2)))
    ms = _time_calls(torch, calls, 3, 1)
    esize = 2 if cfg.dtype == "bf16" else 4
    k_bytes = cfg.H * cfg.L * cfg.d * esize
    n_scores = cfg.H * n * cfg.L
    return {"sampled_rows_per_head": n,
            "predictor_loss": {"ms": round(ms[0], 3), "loss_head0": [round(float(x), 6) for x in res["loss"][0][0].tolist()],
                               "note": "one pass over K (Gram matrix K^T K), the rest is [d, d] / [d, r] algebra in fp64",
                               "k_bytes": k_bytes},
            "profile_sparsity": {"ms": round(ms[1], 3), "sparsity_per_head": [round(float(x), 4) for x in res["prof"][0].tolist()],
                                 "scores_per_sweep": n_scores, "sweeps": 5,
                                 "mfma_tflops": round(5 * 2.0 * cfg.d * n_scores / (ms[1] * 1e-3) / 1e12, 1)}}


def grouping_accuracy(dsv, torch, np, wl, cfg, seed):
    """What sharing the centre query's row costs, on spatially smooth inputs (neighbouring tokens alike, as in
    video latents) and on the benchmark's i.i.d. inputs, at a reduced shape (one head, L = 32768, k = L/16):
    mean fraction of a member's own top-k found in its group's row, and the relative RMS error of the sparse
    outputs (per-query rows, shared rows) against dense attention."""
    from workloads.configs import WorkloadConfig
    grid, cube = (16, 32, 64), (2, 2, 2)
    # predictor of rank r = basis rank: W = G^T (the basis Q and K are built on), which stands for a TRAINED
    # predictor (Q W = Cq G G^T ~ (d/R) Cq, so Q_lr K_lr^T tracks Q K^T); the benchmark's random W selects
    # keys that carry no particular softmax mass, and comparing outputs under it says nothing about grouping
    R = min(cfg.basis_rank, 64)            # the predictor's rank here (the library takes r <= 64)
    c = WorkloadConfig(index=cfg.index, name="grouping_accuracy", B=1, H=1, grid=grid, d=cfg.d, r=R,
                       k=None, k_choices=(), dtype="bf16", basis_rank=R, scale=cfg.scale)
    L, k, G = c.L, c.L // 16, 8
    F, H, W = grid
    res = {}
    for kind in ("smooth", "iid"):
        t = wl.head_tensors_smooth(c, 0, seed=seed, sigma=5.0) if kind == "smooth" else wl.head_tensors(c, 0, seed=seed)
        wq = wk = wl.round_to_dtype(wl.basis(c, seed).T, "bf16")
        td = torch.bfloat16
        dv = {n: torch.from_numpy(t[n]).cuda().to(td)[None, None].contiguous() for n in ("Q", "K", "V")}
        Wq = torch.from_numpy(wq).cuda().to(td)[None].contiguous()
        Wk = torch.from_numpy(wk).cuda().to(td)[None].contiguous()
        p = dsv.Problem(1, 1, L, c.d, c.r, "bf16", [k], c.scale)
        grp = dsv.Grouping(grid, cube)
        idx_q = dsv.lowrank_topk(p, dv["Q"], dv["K"], Wq, Wk).view(L, k)
        idx_g, _, _ = dsv.lowrank_topk_grouped(p, grp, dv["Q"], dv["K"], Wq, Wk, transposed=False)
        # the library's own group-size profiling: overlap per candidate cube, and the largest cube that keeps 80 %
        cubes = [(1, 1, 1), (1, 2, 2), (2, 2, 2), (2, 2, 4), (2, 4, 4), (4, 4, 4)]
        chosen, ov = dsv.choose_grouping(p, grid, cubes, idx_q.reshape(-1), min_overlap=0.8)
        shared = ov[cubes.index(cube)][0]
        Oq, _ = dsv.sparse_attn_fwd(p, dv["Q"], dv["K"], dv["V"], idx_q.reshape(-1))
        Og, _ = dsv.sparse_attn_fwd_grouped(p, grp, dv["Q"], dv["K"], dv["V"], idx_g)
        Od = torch.nn.functional.scaled_dot_product_attention(dv["Q"], dv["K"], dv["V"], scale=c.scale)
        torch.cuda.synchronize()
        rms = lambda x: x.float().pow(2).mean().sqrt().item()
        res[kind] = {"own_topk_found_in_group_row": round(shared, 4),
                     "overlap_by_cube": {"x".join(map(str, cb)): round(ov[i][0], 4) for i, cb in enumerate(cubes)},
                     "largest_cube_keeping_80_percent": list(cubes[chosen]) if chosen >= 0 else None,
                     "rel_rms_error_vs_dense": {"per_query": round(rms(Oq.float() - Od.float()) / rms(Od), 4),
                                                "grouped": round(rms(Og.float() - Od.float()) / rms(Od), 4)}}
        del Od
        del dv, idx_q, idx_g, Oq, Og
        torch.cuda.empty_cache()
    res["shape"] = {"L": L, "k": k, "grid": list(grid), "cube": list(cube), "predictor": f"W = basis^T, rank {c.r}",
                    "smoothing_sigma": 5.0}
    return res


def cpu_baseline(cfg, ks, seed, n_rows, wl, np):
    """Time the CPU oracle (as it stands) on n_rows query rows of head 0 through the whole path and
    scale to the full problem: per-head time = t(project all keys) + (L / n_rows) * t(rows)."""
    import oracle
    t = wl.head_tensors(cfg, 0, seed=seed)
    Wq, Wk = wl.predictor_weights(cfg, 0, seed=seed)
    k = int(ks[0])
    rows = np.linspace(0, cfg.L - 1, n_rows).astype(np.int64)
    t0 = time.perf_counter()
    Klr = oracle.project(t["K"], Wk, cfg.dtype)
    t_keys = time.perf_counter() - t0
    t0 = time.perf_counter()
    Qlr = oracle.project(t["Q"][rows], Wq, cfg.dtype)
    S = oracle.scores(Qlr, Klr)
    idx = oracle.topk_from_scores(S, k)
    t_s1 = time.perf_counter() - t0
    del S
    t0 = time.perf_counter()
    oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], idx, cfg.scale)
    t_fwd = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.sparse_bwd_rows(t["Q"][rows], t["K"], t["V"], idx, t["dO"][rows], cfg.scale)
    t_bwd = time.perf_counter() - t0           # includes the forward it needs for O and lse
    mean_k_scale = float(np.mean(ks)) / k      # other heads scale with their own k in stage 2 only
    total = cfg.H * (t_keys + (cfg.L / n_rows) * (t_s1 + (t_fwd + t_bwd) * mean_k_scale))
    return {"seconds_full_problem_extrapolated": total, "sample_s": t_keys + t_s1 + t_fwd + t_bwd,
            "threads": oracle.max_threads(),
            "parts_s": {"project_keys": t_keys, "stage1_rows": t_s1, "fwd_rows": t_fwd, "bwd_rows": t_bwd}}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one GPU's head-parallel share at the real sequence length); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2502_07590_amd as dsv
    import workloads as wl

    dsv.load_library()  # fails loudly if libdsv.so is missing: there is no fallback
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    if args.dispatcher_table:
        print(json.dumps(dispatcher_table(dsv, torch, np, wl, args)))
        return
    if args.gather_ceiling:
        print(json.dumps(gather_ceiling(dsv, torch)))
        return
    cfg = wl.get_config(args.config)
    ks = wl.k_per_head(cfg, seed=args.seed)
    esize = 2 if cfg.dtype == "bf16" else 4
    n_scores = cfg.H * cfg.L * cfg.L

    t_gen = time.perf_counter()
    g, Wq, Wk = upload_inputs(cfg, args.seed, dev, torch, wl)
    t_gen = time.perf_counter() - t_gen

    if args.calibration_copy_mib:
        src = torch.zeros(args.calibration_copy_mib * (1 << 18), dtype=torch.int32, device=dev)
        dst = torch.add(src, 0)          # one elementwise kernel: reads and writes calibration_copy_mib MiB
        torch.cuda.synchronize()
        del src, dst

    path = Path(dsv, torch, cfg, ks, g, Wq, Wk, sorted_index=not args.unsorted)
    nnz = path.nnz
    ms_per_step, call_ms, kern_ms = path.time(args.steps, args.warmup)

    # ---- derived figures ------------------------------------------------------------------------
    flops_alg = 4.0 * cfg.H * cfg.L * cfg.d * cfg.r + 2.0 * cfg.r * n_scores + 14.0 * cfg.d * nnz
    flops_dense_eq = 14.0 * cfg.d * n_scores
    eff_tflops = flops_dense_eq / (ms_per_step * 1e-3) / 1e12
    # algorithmic bytes per (query, key) pair of each gather pass: one K row + one V row + the index
    # (forward, dq); one Q row + one dO row + the index + lse_i + Delta_i (dkdv)
    pair_bytes = {"sparse_attn_fwd": 2 * cfg.d * esize + 4, "sparse_attn_bwd_dq": 2 * cfg.d * esize + 4,
                  "sparse_attn_bwd_dkdv": 2 * cfg.d * esize + 12}
    pmc_ok = args.config == 2 and not args.unsorted and dsv.version() == PMC_LIBRARY_VERSION
    stage2 = {}
    for n, pb in pair_bytes.items():
        k_ms = kern_ms[SWEEP_OF_CALL[n]]          # the sweep kernel alone, by HIP events on its own stream
        gbs = pb * nnz / (k_ms * 1e-3) / 1e9
        traffic = pmc_traffic_bytes(n) if pmc_ok else None
        stage2[n] = {"bound": "l1", "bound_name": "vector memory path, L2 -> vector L1 -> registers (64 B/clk/CU x 256 CUs x 2.4 GHz)",
                     "achieved": round(gbs, 1), "peak": round(L1_PEAK_GBS, 1), "unit": "GB/s", "frac": round(gbs / L1_PEAK_GBS, 4),
                     "traffic": traffic,
                     "algorithmic_bytes_per_launch": pb * nnz, "kernel": SWEEP_OF_CALL[n] + " kernel of " + n,
                     "kernel_ms": round(k_ms, 3), "call_ms": round(call_ms[n], 3),
                     # the same launch against HBM: the bytes that really crossed the fabric (traffic) per second
                     "hbm": {"achieved": round(traffic / (k_ms * 1e-3) / 1e9, 1) if traffic else None, "peak": HBM_PEAK_GBS,
                             "unit": "GB/s", "frac": round(traffic / (k_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4) if traffic else None,
                             "l2_hit_rate": PMC_CONFIG2[n]["l2_hit_rate"] if pmc_ok else None},
                     "gather_only_ceiling": {"achieved_by_pure_gather_kernel": GATHER_CEILING_GBS[n], "unit": "GB/s",
                                             "frac_of_it": round(gbs / GATHER_CEILING_GBS[n], 4)},
                     "note": "achieved = algorithmic gather bytes (K row + V row + index entry per pair) / kernel time; the ranges "
                             "of the split-K plan stay in each XCD's L2, so the bytes cross the L2 -> L1 path, not HBM"}
    dominant = max(pair_bytes, key=lambda n: kern_ms[SWEEP_OF_CALL[n]])
    roofline = dict(stage2[dominant])
    # Stage 1 is selection work on the plain vector ALUs.  Algorithmic work: per score one compare against the
    # threshold and one update of the selection state = 2 lane-ops per score, ONCE; the implementation recomputes
    # every score in 3 emission sweeps (query-major, 2 key-major) plus 2 (windowed) or 4 (radix) threshold sweeps
    # per head, reported separately.
    s1_ms = call_ms["lowrank_topk_t"]
    s1_lane_ops = 2.0 * n_scores
    sweeps = 3.0 + float(np.mean([2.0 if dsv.threshold_sample_keys(cfg.L, int(k)) else 4.0 for k in ks]))
    s1 = {"bound": "alu", "achieved": round(s1_lane_ops / (s1_ms * 1e-3) / 1e12, 3),
          "peak": round(VALU_LANE_OPS_PER_S / 1e12, 2), "unit": "T lane-ops/s",
          "frac": round(s1_lane_ops / (s1_ms * 1e-3) / VALU_LANE_OPS_PER_S, 4),
          "algorithmic_lane_ops_per_launch": s1_lane_ops, "launch_ms": round(s1_ms, 3),
          "sweeps_over_the_scores": round(sweeps, 2),
          "frac_counting_all_sweeps": round(sweeps * s1_lane_ops / (s1_ms * 1e-3) / VALU_LANE_OPS_PER_S, 4),
          "mfma": {"achieved": round(2.0 * cfg.r * n_scores / (s1_ms * 1e-3) / 1e12, 2), "peak": MFMA_BF16_PEAK_TFLOPS,
                   "unit": "TFLOP/s", "frac": round(2.0 * cfg.r * n_scores / (s1_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4),
                   "achieved_counting_recomputation": round(sweeps * 2.0 * cfg.r * n_scores / (s1_ms * 1e-3) / 1e12, 2)},
          "note": "the score contraction has K = r: 2r flops per score against >= 2 vector-ALU lane-ops per score for the "
                  "selection, so the vector ALUs bound the stage, not the matrix cores (VALU issue 95-104 % busy in the "
                  "threshold and counting sweeps: profiles/config2_pmc_counters.md)"}

    out = {
        "metric": "sparse attention fwd+bwd (stage 1 + stage 2) effective TFLOP/s at L=128k" if args.config == 2
                  else f"sparse attention fwd+bwd effective TFLOP/s, config {args.config}",
        "value": round(eff_tflops, 2), "unit": "TFLOP/s (dense-equivalent: 14*d*H*L^2 / step time)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"config {cfg.index}: {cfg.name}", "B": 1, "H": cfg.H, "L": cfg.L, "d": cfg.d, "r": cfg.r,
                   "k_per_head": sorted(set(ks.tolist())), "nnz_pairs": nnz, "scale": cfg.scale, "seed": args.seed,
                   "sorted_index_flag": not args.unsorted},
        "stage_ms": {n: round(v, 3) for n, v in call_ms.items()},
        "kernel_ms": {n: round(v, 3) for n, v in kern_ms.items()},
        "algorithmic_tflops": round(flops_alg / (ms_per_step * 1e-3) / 1e12, 2),
        "input_generation_s": round(t_gen, 1),
        "roofline": roofline,
        "stage_rooflines": dict(stage2, lowrank_topk_t=s1),
    }

    # ---- dense comparator: library flash attention fwd+bwd at the same shape ----------------------
    dense_ms = None
    if not args.no_dense:
        try:
            import torch.nn.functional as F
            q = g["Q"].clone().requires_grad_(True); k_ = g["K"].clone().requires_grad_(True); v = g["V"].clone().requires_grad_(True)
            def dense():
                o = F.scaled_dot_product_attention(q, k_, v, scale=cfg.scale)
                o.backward(g["dO"])
                q.grad = k_.grad = v.grad = None
            dense()
            dense()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            reps = 2
            e0.record()
            for _ in range(reps):
                dense()
            e1.record()
            torch.cuda.synchronize()
            dense_ms = e0.elapsed_time(e1) / reps
            out["dense"] = {"impl": "torch scaled_dot_product_attention fwd+bwd", "ms": round(dense_ms, 3),
                            "tflops": round(flops_dense_eq / (dense_ms * 1e-3) / 1e12, 2),
                            "speedup_sparse_over_dense": round(dense_ms / ms_per_step, 3)}
            del q, k_, v
        except Exception as e:  # the comparator is optional context; the sparse path above is the product
            out["dense"] = {"error": repr(e)[:200]}

    # ---- whole path at other densities, same shape (the table a dispatcher would consume) -----------
    if args.density_sweep:
        del path
        torch.cuda.empty_cache()
        sweep = []
        for frac in (0.005, 0.01, 0.02, 0.03125, 0.0625, 0.10, 0.125):
            kk = max(1, int(round(cfg.L * frac)))
            pth = Path(dsv, torch, cfg, [kk] * cfg.H, g, Wq, Wk, sorted_index=not args.unsorted)
            ms, cms, _ = pth.time(2, 1)
            sweep.append({"density": frac, "k": kk, "ms_per_step": round(ms, 2), "stage1_ms": round(cms["lowrank_topk_t"], 2),
                          "stage2_ms": round(ms - cms["lowrank_topk_t"], 2),
                          "speedup_over_dense": round(dense_ms / ms, 3) if dense_ms else None})
            del pth
            torch.cuda.empty_cache()
        out["density_sweep"] = sweep
        if dense_ms:
            out["crossover_density"] = interpolate_crossover([(s_["density"], s_["ms_per_step"]) for s_ in sweep], dense_ms)

    # ---- query-grouped variant (the paper's answer to the per-query gather cost) --------------------
    # both extras are reported next to the headline; they never change `value`
    extras_ok = cfg.dtype == "bf16" and cfg.d == 128 and all(x % 2 == 0 for x in cfg.grid)
    if extras_ok and not args.no_grouped:   # the grouped backward's workspace must fit beside what is resident
        p_g = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, [int(k) for k in ks], cfg.scale, sorted_index=True)
        need = dsv.sparse_attn_bwd_grouped_workspace(p_g, dsv.Grouping(cfg.grid, (2, 2, 2))) + 3 * p_g.nnz + 8 * g["Q"].numel() * 2
        if need > 0.8 * torch.cuda.mem_get_info()[1]:
            args.no_grouped = True
            out["grouped"] = {"skipped": f"needs about {need / 1e9:.0f} GB"}
    if (extras_ok and not args.no_grouped) or args.grouped or args.grouped_density_sweep:
        try:
            del path
        except NameError:
            pass
        torch.cuda.empty_cache()
        out["grouped"] = grouped_report(dsv, torch, np, wl, cfg, ks, g, Wq, Wk, max(args.steps, 2), 1, dense_ms, ms_per_step)
        # the grouped step at other densities (same shape, uniform k) and where it meets dense attention
        gsweep = []
        for frac in ((0.03125, 0.0625, 0.10, 0.125, 0.1875, 0.25) if args.grouped_density_sweep else ()):
            kk = max(1, int(round(cfg.L * frac)))
            r = grouped_report(dsv, torch, np, wl, cfg, [kk] * cfg.H, g, Wq, Wk, 2, 1, dense_ms, ms_per_step)
            gsweep.append({"density": frac, "k": kk, "ms_per_step": r["ms_per_step"], "stage_ms": r["stage_ms"],
                           "speedup_over_dense": r["speedup_over_dense"]})
            print(json.dumps(gsweep[-1]), file=sys.stderr, flush=True)
        if args.grouped_cubes:
            out["grouped"]["other_cubes"] = []
            for cube in ((2, 2, 4), (2, 4, 4)):
                r = grouped_report(dsv, torch, np, wl, cfg, ks, g, Wq, Wk, 2, 1, dense_ms, ms_per_step, cube=cube)
                out["grouped"]["other_cubes"].append({k_: r[k_] for k_ in ("cube", "G", "ms_per_step", "kernel_ms", "stage_ms",
                                                                           "speedup_over_dense")})
                print(json.dumps(out["grouped"]["other_cubes"][-1]), file=sys.stderr, flush=True)
        if gsweep:
            out["grouped"]["density_sweep"] = gsweep
        if gsweep and dense_ms:
            out["grouped"]["crossover_density"] = interpolate_crossover([(s_["density"], s_["ms_per_step"]) for s_ in gsweep], dense_ms)
        out["grouped"]["accuracy"] = grouping_accuracy(dsv, torch, np, wl, cfg, args.seed)

    if (extras_ok and not args.no_predictor) or args.predictor:
        out["predictor_side"] = predictor_report(dsv, torch, cfg, ks, g, Wq, Wk)

    # ---- CPU oracle timed on a bounded sample ------------------------------------------------------
    if not args.no_cpu_baseline:
        import oracle
        threads = oracle.max_threads()
        n_rows = args.cpu_rows or max(threads * 128, 256)
        cb = cpu_baseline(cfg, ks, args.seed, n_rows, wl, np)
        out["cpu_baseline"] = {
            "value": round(flops_dense_eq / cb["seconds_full_problem_extrapolated"] / 1e12, 6),
            "unit": out["unit"], "cores": cb["threads"], "kind": "oracle",
            "sample": f"{n_rows} evenly spaced query rows of head 0 through projection, scoring, selection, sparse "
                      f"forward and backward ({cb['sample_s']:.1f} s measured), scaled by L/{n_rows} per head and by "
                      f"{cfg.H} heads (extrapolated full problem: {cb['seconds_full_problem_extrapolated']:.0f} s)",
            "parts_s": {k_: round(v, 3) for k_, v in cb["parts_s"].items()},
        }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
