"""Pins of the oracle's predictor-side routines (paper Sec. "Low-Rank based Sparsity Prediction": the
0.95 cosine + 0.05 norm approximation loss on sampled queries; Sec. "Sparsity Profiling" / "Exploiting Dynamic
Sparsity": sparsity of a head from the keys that hold 90 % of each sampled query's softmax)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from workloads.configs import WorkloadConfig


def _cfg(L, d=64, r=16, R=32):
    return WorkloadConfig(index=400, name="predictor_case", B=1, H=1, grid=(1, 1, L), d=d, r=r, k=None, k_choices=(),
                          dtype="f32", basis_rank=R, scale=1.0 / np.sqrt(d))


def _torch_loss(Qs, K, Wq, Wk):
    A = Qs @ K.T
    Ah = (Qs @ Wq) @ (K @ Wk).T
    cos = (1.0 - torch.nn.functional.cosine_similarity(Ah, A, dim=1)).mean()
    norm = torch.nn.functional.mse_loss(Ah, A)
    return 0.95 * cos + 0.05 * norm, cos, norm


@pytest.mark.parametrize("L,n,d,r", [(96, 7, 64, 16), (257, 33, 32, 8)])
def test_loss_and_gradients_match_torch_autograd(L, n, d, r):
    cfg = _cfg(L, d, r)
    t = wl.head_tensors(cfg, 0, names=("Q", "K"))
    Wq, Wk = wl.predictor_weights(cfg, 0)
    rows = np.linspace(0, L - 1, n).astype(np.int64)
    (loss, cos, norm), dWq, dWk = oracle.predictor_loss(t["Q"][rows], t["K"], Wq, Wk)
    tq, tk = torch.tensor(t["Q"][rows], dtype=torch.float64), torch.tensor(t["K"], dtype=torch.float64)
    twq = torch.tensor(Wq, dtype=torch.float64, requires_grad=True)
    twk = torch.tensor(Wk, dtype=torch.float64, requires_grad=True)
    l, c, m = _torch_loss(tq, tk, twq, twk)
    l.backward()
    assert abs(loss - l.item()) < 1e-12 * max(1.0, abs(l.item()))
    assert abs(cos - c.item()) < 1e-12 and abs(norm - m.item()) < 1e-10 * max(1.0, m.item())
    assert np.abs(dWq - twq.grad.numpy()).max() < 1e-10 * max(1.0, np.abs(dWq).max())
    assert np.abs(dWk - twk.grad.numpy()).max() < 1e-10 * max(1.0, np.abs(dWk).max())


def test_loss_closed_forms_and_finite_differences():
    cfg = _cfg(64, d=32, r=32)
    t = wl.head_tensors(cfg, 0, names=("Q", "K"))
    rows = np.arange(0, 64, 5)
    eye = np.eye(32, dtype=np.float32)
    # identity predictor: the approximation is exact -> both terms vanish, and so does the gradient of the norm term
    (loss, cos, norm), dWq, dWk = oracle.predictor_loss(t["Q"][rows], t["K"], eye, eye)
    assert abs(cos) < 1e-14 and norm < 1e-20 and abs(loss) < 1e-14
    assert np.abs(dWq).max() < 1e-8 and np.abs(dWk).max() < 1e-8
    # a predictor scaled by c: cosine unchanged (0), norm term = (c^2 - 1)^2 * mean(a^2)
    c = 1.5
    (_, cos2, norm2), _, _ = oracle.predictor_loss(t["Q"][rows], t["K"], c * eye, c * eye)
    A = t["Q"][rows].astype(np.float64) @ t["K"].astype(np.float64).T
    assert abs(cos2) < 1e-14 and abs(norm2 - (c * c - 1.0) ** 2 * (A * A).mean()) < 1e-9 * norm2
    # the negated predictor on one side: cosine -1 -> CosLoss = 2
    (_, cos3, _), _, _ = oracle.predictor_loss(t["Q"][rows], t["K"], -eye, eye)
    assert abs(cos3 - 2.0) < 1e-14
    # central finite differences on a random predictor
    cfg2 = _cfg(48, d=32, r=4)
    t2 = wl.head_tensors(cfg2, 0, names=("Q", "K"))
    Wq, Wk = wl.predictor_weights(cfg2, 0)
    rows2 = np.arange(0, 48, 4)
    (l0, _, _), dWq, dWk = oracle.predictor_loss(t2["Q"][rows2], t2["K"], Wq, Wk)
    eps = 2.0 ** -12
    rng = np.random.default_rng(1)
    for which, grad in ((0, dWq), (1, dWk)):
        for _ in range(5):
            a, b = int(rng.integers(32)), int(rng.integers(4))
            Wp, Wm = [Wq.copy(), Wk.copy()], [Wq.copy(), Wk.copy()]
            Wp[which][a, b] += eps; Wm[which][a, b] -= eps
            fd = (oracle.predictor_loss(t2["Q"][rows2], t2["K"], *Wp)[0][0] -
                  oracle.predictor_loss(t2["Q"][rows2], t2["K"], *Wm)[0][0]) / (2 * eps)
            assert abs(fd - grad[a, b]) < 1e-6 * max(1.0, abs(grad[a, b])), (which, a, b, fd, grad[a, b])


def test_profile_sparsity_against_a_sort_in_numpy_and_closed_forms():
    cfg = _cfg(512, d=64)
    t = wl.head_tensors(cfg, 0, names=("Q", "K"))
    rows = np.arange(3, 512, 37)
    s, counts = oracle.profile_sparsity(t["Q"][rows], t["K"], cfg.scale * 4.0, 0.9)
    S = cfg.scale * 4.0 * (t["Q"][rows].astype(np.float64) @ t["K"].astype(np.float64).T)
    P = np.exp(S - S.max(axis=1, keepdims=True)); P /= P.sum(axis=1, keepdims=True)
    want = np.array([int(np.searchsorted(np.cumsum(np.sort(p)[::-1]), 0.9) + 1) for p in P])
    assert np.abs(counts - want).max() <= 1 and (counts == want).mean() > 0.9      # cumulative sums in another order
    assert abs(s - np.mean(1.0 - counts / 512.0)) < 1e-15
    # uniform attention (Q = 0): ceil(0.9 L) keys are needed -> sparsity 1 - ceil(0.9 L) / L
    s0, c0 = oracle.profile_sparsity(np.zeros((3, 64), dtype=np.float32), t["K"], 1.0, 0.9)
    assert np.all(c0 == int(np.ceil(0.9 * 512 - 1e-9))) and abs(s0 - (1.0 - c0[0] / 512.0)) < 1e-15
    # one dominant key: a single critical key
    Kd = t["K"].copy(); q = np.zeros((1, 64), dtype=np.float32); q[0, 0] = 50.0; Kd[:, 0] = 0.0; Kd[17, 0] = 1.0
    s1, c1 = oracle.profile_sparsity(q, Kd, 1.0, 0.9)
    assert c1[0] == 1 and abs(s1 - (1.0 - 1.0 / 512.0)) < 1e-15
    # the synthetic recipe's regime: a few per cent of the keys hold 90 % of the mass at logit std 2.83
    cfg1 = WorkloadConfig(index=1, name="c1", B=1, H=1, grid=(1, 1, 4096), d=128, r=16, k=None, k_choices=(), dtype="bf16",
                          basis_rank=64, scale=2.0 / np.sqrt(128))
    t1 = wl.head_tensors(cfg1, 0, names=("Q", "K"))
    s2, _ = oracle.profile_sparsity(t1["Q"][::256], t1["K"], cfg1.scale, 0.9)
    assert 0.90 < s2 < 0.99, s2        # (a closed form for Gaussian logits gives 0.94; the products of Gaussians are heavier-tailed)


def test_ema():
    assert oracle.ema(0.5, 1.0, 0.25) == 0.625
    assert oracle.ema(0.7, 0.7, 0.1) == pytest.approx(0.7, abs=1e-16)
