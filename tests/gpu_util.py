"""Helpers shared by the GPU parity tests: build a seeded case, move it to the device."""
from __future__ import annotations

import math

import numpy as np
import torch

import workloads as wl
from workloads.configs import WorkloadConfig

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def make_cfg(L, d, r, H, dtype, basis_rank=32, scale_num=1.0, k=None, index=100):
    return WorkloadConfig(index=index, name=f"case_L{L}", B=1, H=H, grid=(1, 1, L), d=d, r=r, k=k, k_choices=(),
                          dtype=dtype, basis_rank=basis_rank, scale=scale_num / math.sqrt(d))


class Case:
    """All heads of one seeded problem, on the host (float32 holders) and on the device."""

    def __init__(self, cfg, ks, seed=0, device="cuda:0", names=("Q", "K", "V", "dO")):
        self.cfg, self.ks = cfg, [int(x) for x in ks]
        self.host = {n: [] for n in names}
        self.Wq, self.Wk = [], []
        for h in range(cfg.H):
            t = wl.head_tensors(cfg, h, seed=seed, names=names)
            for n in names:
                self.host[n].append(t[n])
            wq, wk = wl.predictor_weights(cfg, h, seed=seed)
            self.Wq.append(wq)
            self.Wk.append(wk)
        td = TORCH_DTYPE[cfg.dtype]
        self.dev = {n: torch.from_numpy(np.stack(v)[None]).to(device).to(td).contiguous() for n, v in self.host.items()}
        self.dWq = torch.from_numpy(np.stack(self.Wq)).to(device).to(td).contiguous()
        self.dWk = torch.from_numpy(np.stack(self.Wk)).to(device).to(td).contiguous()
        self.off = wl.idx_offsets(1, cfg.H, cfg.L, self.ks)

    def problem(self, dsv, sorted_index=False):
        c = self.cfg
        return dsv.Problem(1, c.H, c.L, c.d, c.r, c.dtype, self.ks, c.scale, sorted_index=sorted_index)

    def idx_rows(self, idx_flat: np.ndarray, h: int) -> np.ndarray:
        return idx_flat[self.off[h]:self.off[h + 1]].reshape(self.cfg.L, self.ks[h])


def tolerance(dtype: str, ref: np.ndarray) -> np.ndarray:
    """Element-wise error allowed against the fp64 oracle: max-abs 2e-2 (bf16) / 1e-4 (fp32), widened
    to a few output ulps where the reference value itself is large."""
    if dtype == "bf16":
        return np.maximum(2e-2, 2.0 ** -7 * np.abs(ref))
    return np.maximum(1e-4, 2.0 ** -20 * np.abs(ref))


def assert_close(name, got: torch.Tensor, ref: np.ndarray, dtype: str):
    g = got.detach().to(torch.float64).cpu().numpy().reshape(ref.shape)
    err = np.abs(g - ref)
    tol = tolerance(dtype, ref)
    bad = err > tol
    assert not bad.any(), (f"{name}: {bad.sum()} of {bad.size} elements out of tolerance; max abs err "
                           f"{err.max():.3e} at ref {ref.flat[err.argmax()]:.3e}")
    return float(err.max())


def score_error_bound(Qlr_dev_rows: np.ndarray, Klr_dev: np.ndarray, S_dev_exact: np.ndarray, S_or: np.ndarray,
                      r: int) -> np.ndarray:
    """e[a, j] >= |S_device[a, j] - S_oracle[a, j]| for device scores accumulated in fp32:

        e = r * 2^-23 * sum_t |q~_t k~_t|   +   |sum_t q~_t k~_t  -  sum_t q_t k_t|

    q~, k~: the device's projections (each within one storage ulp of the oracle's q, k -- the projection
    test asserts that); the first term bounds the fp32 accumulation of the r products, the second is the
    exact effect of projected terms that were rounded the other way (zero where the projections agree).
    S_dev_exact = exact scores of the device's projections, S_or = exact scores of the oracle's."""
    absprod = np.abs(Qlr_dev_rows).astype(np.float64) @ np.abs(Klr_dev).astype(np.float64).T
    return r * 2.0 ** -23 * absprod + np.abs(S_dev_exact - S_or) + 1e-300


def assert_t3_valid(name: str, got_row: np.ndarray, ref_row: np.ndarray, S_or_row: np.ndarray, e_row: np.ndarray,
                    k: int) -> bool:
    """Tier T3: the device's index row against the pure fp64 oracle's.  Both are exact top-k sets of their
    own score rows, which differ by at most e_row element-wise, so the k-th largest values differ by at most
    max(e_row) and every key j in the symmetric difference satisfies
        |S_oracle[j] - tau_oracle| <= max_j' e[j'] + e[j].
    Returns True when the rows are identical."""
    if np.array_equal(got_row, ref_row):
        return True
    L = S_or_row.shape[0]
    tau = np.partition(S_or_row, L - k)[L - k]              # the oracle's k-th largest score
    sym = np.setxor1d(got_row, ref_row)
    eps = e_row.max() + e_row[sym]
    dist = np.abs(S_or_row[sym] - tau)
    assert np.all(dist <= eps), (f"{name}: {int((dist > eps).sum())} of {sym.size} differing keys lie outside the "
                                 f"rounding band of the threshold (worst {dist.max():.3e} vs eps {eps.max():.3e})")
    return False
