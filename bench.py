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

# L2 -> fabric traffic of the stage-2 kernels at config 2, bytes per launch, from two rocprofv3 --pmc
# runs (FETCH_SIZE, WRITE_SIZE, in KiB), each scaled by what the same counter reads for a plain 1 GiB
# elementwise copy in the same run (FETCH_SIZE reads 0.5 GiB for it: factor 2.0; WRITE_SIZE reads
# 1 GiB: factor 1.0).  See profiles/stage2_config2_pmc_traffic.md.
PMC_TRAFFIC_CONFIG2 = {
    "sparse_attn_fwd": int((31044477 * 2.0 + 14155840 * 1.0) * 1024),
    "sparse_attn_bwd_dq": int((48443068 * 2.0 + 12976310 * 1.0) * 1024),
    "sparse_attn_bwd_dkdv": int((34221672 * 2.0 + 12582937 * 1.0) * 1024),
}
# the gather sweep inside each stage-2 call (the kernel the roofline object is about)
SWEEP_OF_CALL = {"sparse_attn_fwd": "fwd_sweep", "sparse_attn_bwd_dq": "dq_sweep", "sparse_attn_bwd_dkdv": "dkdv_sweep"}
L1_PEAK_GBS = 256 * 64 * 2.4          # 256 CUs x 64 B per clock (vector L1 -> registers) x 2.4 GHz


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
    stage2 = {}
    for n, pb in pair_bytes.items():
        k_ms = kern_ms[SWEEP_OF_CALL[n]]          # the sweep kernel alone, by HIP events on its own stream
        gbs = pb * nnz / (k_ms * 1e-3) / 1e9
        stage2[n] = {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4),
                     "traffic": PMC_TRAFFIC_CONFIG2.get(n) if (args.config == 2 and not args.unsorted) else None,
                     "algorithmic_bytes_per_launch": pb * nnz, "kernel": SWEEP_OF_CALL[n] + " kernel of " + n,
                     "kernel_ms": round(k_ms, 3), "call_ms": round(call_ms[n], 3),
                     # the requested bytes are served by L2 and the vector L1, not by HBM (see traffic): the
                     # path that bounds the kernel is L1 -> registers, 64 B per clock per CU
                     "l1_path": {"peak": round(L1_PEAK_GBS, 1), "unit": "GB/s", "frac": round(gbs / L1_PEAK_GBS, 4)},
                     "note": "achieved counts the bytes the gathers request; they are served from L2 (compare "
                             "traffic, the bytes that crossed the fabric), so frac against the HBM peak exceeds 1; "
                             "l1_path is the same rate against the L2 -> L1 -> register path that bounds the kernel"}
    dominant = max(pair_bytes, key=lambda n: kern_ms[SWEEP_OF_CALL[n]])
    roofline = dict(stage2[dominant])
    # stage 1 is selection work on plain VALU lanes: per score at least one subtract/compare and one
    # mask update in each of its passes (4 threshold passes + emit + 2 key-major passes = 7)
    s1_lane_ops = 2.0 * 7 * n_scores
    s1 = {"bound": "alu", "achieved": round(s1_lane_ops / (call_ms["lowrank_topk_t"] * 1e-3) / 1e12, 3),
          "peak": round(VALU_LANE_OPS_PER_S / 1e12, 2), "unit": "T lane-ops/s",
          "frac": round(s1_lane_ops / (call_ms["lowrank_topk_t"] * 1e-3) / VALU_LANE_OPS_PER_S, 4),
          "algorithmic_lane_ops_per_launch": s1_lane_ops, "launch_ms": round(call_ms["lowrank_topk_t"], 3),
          "mfma_tflops": round(2.0 * cfg.r * n_scores * 7 / (call_ms["lowrank_topk_t"] * 1e-3) / 1e12, 2)}

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
            below = [s for s in sweep if s["ms_per_step"] <= dense_ms]
            out["crossover_density"] = max(s["density"] for s in below) if below else None

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
