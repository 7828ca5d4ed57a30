"""GPU parity of the predictor side (dsv_predictor_loss) against the CPU oracle, through the C ABI."""
import math

import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads.configs import WorkloadConfig

pytestmark = pytest.mark.gpu

dsv = pytest.importorskip("paper_2502_07590_amd")


def _cfg(L, d, r, dtype, H=2, R=32):
    return WorkloadConfig(index=500, name="predictor_gpu", B=1, H=H, grid=(1, 1, L), d=d, r=r, k=None, k_choices=(),
                          dtype=dtype, basis_rank=R, scale=1.0 / math.sqrt(d))


@pytest.mark.parametrize("L,d,r,dtype,n", [(1024, 64, 16, "f32", 64), (3000, 128, 16, "bf16", 187), (2050, 128, 64, "bf16", 33),
                                           (700, 64, 32, "bf16", 700)])
def test_predictor_loss_and_gradients_match_oracle(L, d, r, dtype, n):
    cfg = _cfg(L, d, r, dtype)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    t = [wl.head_tensors(cfg, h, names=("Q", "K")) for h in range(cfg.H)]
    W = [wl.predictor_weights(cfg, h) for h in range(cfg.H)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()
    Q, K = dev(np.stack([x["Q"] for x in t]))[None], dev(np.stack([x["K"] for x in t]))[None]
    Wq, Wk = dev(np.stack([w[0] for w in W])), dev(np.stack([w[1] for w in W]))
    rows = np.sort(np.random.default_rng(3).choice(L, size=n, replace=False)).astype(np.int32)
    p = dsv.Problem(1, cfg.H, L, d, r, dtype, [1] * cfg.H, cfg.scale)
    loss, dWq, dWk = dsv.predictor_loss(p, Q, K, Wq, Wk, torch.from_numpy(rows).cuda())
    torch.cuda.synchronize()
    loss, dWq, dWk = loss.cpu().numpy().astype(np.float64), dWq.cpu().numpy().astype(np.float64), dWk.cpu().numpy().astype(np.float64)
    for h in range(cfg.H):
        ref, rWq, rWk = oracle.predictor_loss(t[h]["Q"][rows], t[h]["K"], W[h][0], W[h][1])
        # the device forms the same quantities from the fp32-accumulated Gram matrix K^T K (relative 1e-5) in fp64,
        # and returns fp32: 1e-4 relative to the largest entry covers both
        for name, got, want in (("loss", loss[h], np.array(ref)), ("dWq", dWq[h], rWq), ("dWk", dWk[h], rWk)):
            tol = 1e-4 * max(np.abs(want).max(), 1e-30)
            assert np.abs(got - want).max() <= tol, f"{name}[h={h}]: {np.abs(got - want).max():.3e} > {tol:.3e}"


def test_identity_predictor_has_zero_loss():
    L, d = 512, 64
    cfg = _cfg(L, d, 64, "f32", H=1)
    t = wl.head_tensors(cfg, 0, names=("Q", "K"))
    eye = torch.eye(64, device="cuda")[None].contiguous()
    Q, K = torch.from_numpy(t["Q"]).cuda()[None, None].contiguous(), torch.from_numpy(t["K"]).cuda()[None, None].contiguous()
    p = dsv.Problem(1, 1, L, d, 64, "f32", [1], cfg.scale)
    loss, dWq, dWk = dsv.predictor_loss(p, Q, K, eye, eye, torch.arange(0, L, 16, dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    assert abs(float(loss[0, 1])) < 1e-5 and abs(float(loss[0, 2])) < 1e-3 * float((Q[0, 0] @ K[0, 0].T).pow(2).mean())


@pytest.mark.parametrize("L,d,dtype,n,scale_mul", [(1024, 64, "f32", 40, 4.0), (4096, 128, "bf16", 100, 2.0), (3001, 128, "bf16", 33, 2.0)])
def test_profile_sparsity_matches_oracle(L, d, dtype, n, scale_mul):
    cfg = _cfg(L, d, 16, dtype, R=64 if d == 128 else 32)
    td = torch.bfloat16 if dtype == "bf16" else torch.float32
    t = [wl.head_tensors(cfg, h, names=("Q", "K")) for h in range(cfg.H)]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda().to(td).contiguous()
    Q, K = dev(np.stack([x["Q"] for x in t]))[None], dev(np.stack([x["K"] for x in t]))[None]
    rows = np.sort(np.random.default_rng(5).choice(L, size=n, replace=False)).astype(np.int32)
    scale = scale_mul / math.sqrt(d)
    p = dsv.Problem(1, cfg.H, L, d, 16, dtype, [1] * cfg.H, scale)
    ema = torch.full((cfg.H,), 0.5, dtype=torch.float32, device="cuda")
    sparsity, counts = dsv.profile_sparsity(p, Q, K, torch.from_numpy(rows).cuda(), mass=0.9, ema=ema, alpha=0.25)
    torch.cuda.synchronize()
    sparsity, counts, ema = sparsity.cpu().numpy(), counts.cpu().numpy(), ema.cpu().numpy()
    for h in range(cfg.H):
        s_ref, c_ref = oracle.profile_sparsity(t[h]["Q"][rows], t[h]["K"], scale, 0.9)
        # the device sums fp32 probabilities in another order: where the cumulative mass passes 0.9 within rounding
        # of a key boundary the count moves by one key
        diff = np.abs(counts[h].astype(np.int64) - c_ref)
        assert diff.max() <= 1 and (diff == 0).mean() > 0.8, (diff.max(), (diff == 0).mean())
        assert abs(sparsity[h] - s_ref) <= 1.0 / L + 1e-6
        assert abs(ema[h] - oracle.ema(0.5, float(sparsity[h]), 0.25)) < 1e-6
