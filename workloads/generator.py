"""Seeded generators for every tensor the tests and the benchmark feed to the path.

Recipe (one function family, all configs):
  * a Gaussian basis G [R, d], entries N(0, 1/R), shared by Q and K and by all
    heads of a config;
  * per head, coefficient matrices Cq, Ck [L, R] ~ N(0, 1) drawn independently;
    Q = Cq G + 0.1 N(0,1), K = Ck G + 0.1 N(0,1); V, dO ~ N(0, 1);
  * predictor weights Wq, Wk [d, r] ~ N(0, 1/d), one pair per head;
  * everything is drawn in fp32/fp64, then rounded once to the config's
    storage dtype and returned as float32 arrays that hold exactly the rounded
    values (a bf16 value is a float32 whose low 16 mantissa bits are zero).

Every stream is keyed by (seed, config index, tensor id, head), so a test can
draw one head, or one tensor, without drawing the rest.  Nothing here computes
any part of the attention method.
"""
from __future__ import annotations

import numpy as np

from .configs import WorkloadConfig

_TENSOR_ID = {"basis": 1, "Q": 2, "K": 3, "V": 4, "dO": 5, "Wq": 6, "Wk": 7,
              "k_per_head": 8, "subset_idx": 9, "progression": 10, "ternary": 11, "tokens": 12}


def _rng(seed: int, cfg_index: int, tensor: str, head: int = 0, extra: int = 0):
    return np.random.default_rng([int(seed), int(cfg_index), _TENSOR_ID[tensor], int(head), int(extra)])


def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round an array to the storage dtype; the result is float32 holding the rounded values.

    "f32": plain cast.  "bf16": round-to-nearest-even on the upper 16 bits of the
    float32 pattern (inputs are finite, so no NaN handling is needed).
    """
    x32 = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x32
    if dtype != "bf16":
        raise ValueError(f"unknown dtype {dtype!r}")
    u = x32.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    u = (u & 0xFFFF0000).astype(np.uint32)
    return u.view(np.float32).reshape(x32.shape)


def basis(cfg: WorkloadConfig, seed: int = 0) -> np.ndarray:
    """G [R, d] float64, entries N(0, 1/R)."""
    g = _rng(seed, cfg.index, "basis").standard_normal((cfg.basis_rank, cfg.d))
    return g / np.sqrt(cfg.basis_rank)


def head_tensors(cfg: WorkloadConfig, head: int, seed: int = 0, names=("Q", "K", "V", "dO"),
                 rows: slice | None = None) -> dict:
    """Draw the named tensors of one head, each [L, d] float32 holding dtype-rounded values.

    `rows` (a slice) returns only those token rows; the full stream is still drawn so
    that the values do not depend on which rows are asked for.
    """
    out = {}
    L, d, R = cfg.L, cfg.d, cfg.basis_rank
    G = None
    for name in names:
        rng = _rng(seed, cfg.index, name, head)
        if name in ("Q", "K"):
            if G is None:
                G = basis(cfg, seed)
            coef = rng.standard_normal((L, R))
            noise = rng.standard_normal((L, d), dtype=np.float32)
            x = (coef @ G).astype(np.float32) + np.float32(0.1) * noise
        elif name in ("V", "dO"):
            x = rng.standard_normal((L, d), dtype=np.float32)
        else:
            raise ValueError(name)
        x = round_to_dtype(x, cfg.dtype)
        out[name] = x if rows is None else np.ascontiguousarray(x[rows])
    return out


def predictor_weights(cfg: WorkloadConfig, head: int, seed: int = 0):
    """(Wq, Wk), each [d, r] float32 holding dtype-rounded N(0, 1/d) values."""
    ws = []
    for name in ("Wq", "Wk"):
        w = _rng(seed, cfg.index, name, head).standard_normal((cfg.d, cfg.r)) / np.sqrt(cfg.d)
        ws.append(round_to_dtype(w, cfg.dtype))
    return ws[0], ws[1]


def k_per_head(cfg: WorkloadConfig, seed: int = 0) -> np.ndarray:
    """int32 [H]: KV kept per query for each head (one sparsity level per head)."""
    if cfg.k is not None:
        return np.full(cfg.H, cfg.k, dtype=np.int32)
    choice = _rng(seed, cfg.index, "k_per_head").integers(0, len(cfg.k_choices), size=cfg.H)
    return np.asarray(cfg.k_choices, dtype=np.int32)[choice]


def idx_offsets(B: int, H: int, L: int, ks) -> np.ndarray:
    """int64 [B*H+1]: element offset of each (batch, head) block of the ragged index tensor."""
    ks = np.asarray(ks, dtype=np.int64)
    per = np.tile(ks * np.int64(L), B)
    off = np.zeros(B * H + 1, dtype=np.int64)
    np.cumsum(per, out=off[1:])
    return off


def random_subset_idx(L: int, k: int, n_rows: int, seed: int = 0, head: int = 0,
                      ascending: bool = True) -> np.ndarray:
    """int32 [n_rows, k]: a uniformly random k-subset of [0, L) per row."""
    rng = _rng(seed, 0, "subset_idx", head, extra=L * 131 + k)
    keys = rng.random((n_rows, L))
    idx = np.argpartition(keys, k - 1, axis=1)[:, :k] if k < L else np.tile(np.arange(L), (n_rows, 1))
    if ascending:
        idx = np.sort(idx, axis=1)
    else:
        idx = rng.permuted(idx, axis=1)
    return np.ascontiguousarray(idx, dtype=np.int32)


# ---------------------------------------------------------------------------------------
# Arithmetic-progression index sets: a valid (distinct, in range) index tensor of any size
# whose rows AND columns can be written down in closed form, so that sampled rows of
# dK/dV can be checked at full problem size without scanning tens of GB of indices.
# Row i holds { (base_i + t * g_i) mod L : 0 <= t < k } with g_i odd and L a power of two.
# ---------------------------------------------------------------------------------------

def _inv_mod_pow2(g: np.ndarray, L: int) -> np.ndarray:
    g = g.astype(np.uint64)
    x = g.copy()
    two = np.uint64(2)
    with np.errstate(over="ignore"):
        for _ in range(6):
            x = x * (two - g * x)
    return (x & np.uint64(L - 1)).astype(np.int64)


def progression_params(L: int, seed: int = 0, head: int = 0):
    """(base [L], g [L], ginv [L]) int64; g odd, ginv = g^-1 mod L.  L must be a power of two."""
    if L & (L - 1):
        raise ValueError("progression index sets need L to be a power of two")
    rng = _rng(seed, 0, "progression", head, extra=L)
    base = rng.integers(0, L, size=L, dtype=np.int64)
    g = rng.integers(0, max(L // 2, 1), size=L, dtype=np.int64) * 2 + 1
    return base, g, _inv_mod_pow2(g, L)


def progression_idx_rows(L: int, k: int, rows, params) -> np.ndarray:
    """int32 [len(rows), k], ascending: the index rows of the given queries."""
    base, g, _ = params
    rows = np.asarray(rows, dtype=np.int64)
    t = np.arange(k, dtype=np.int64)[None, :]
    idx = (base[rows, None] + t * g[rows, None]) & (L - 1)
    return np.sort(idx, axis=1).astype(np.int32)


def progression_queries_of_key(L: int, k: int, key: int, params) -> np.ndarray:
    """int64 [*], ascending: every query i whose index row contains `key`."""
    base, g, ginv = params
    t = ((np.int64(key) - base) * ginv) & (L - 1)
    return np.nonzero(t < k)[0].astype(np.int64)


def ternary_head_tensors(L: int, d: int, r: int, seed: int = 0, head: int = 0):
    """Q, K [L, d] and Wq, Wk [d, r] with entries in {-1, 0, 1} (float32).

    With such inputs every projected value is an integer of magnitude <= d and every
    low-rank score an integer of magnitude <= r d^2 < 2^24: exact in bf16 / fp32 whatever
    the summation order, and full of ties.
    """
    rng = _rng(seed, 0, "ternary", head, extra=L * 7 + d * 3 + r)
    Q = rng.integers(-1, 2, size=(L, d)).astype(np.float32)
    K = rng.integers(-1, 2, size=(L, d)).astype(np.float32)
    Wq = rng.integers(-1, 2, size=(d, r)).astype(np.float32)
    Wk = rng.integers(-1, 2, size=(d, r)).astype(np.float32)
    return Q, K, Wq, Wk


# ---------------------------------------------------------------------------------------
# Spatially smooth variant: video latents are continuous signals, so neighbouring tokens of
# the frames x height x width grid have similar queries and keys (the i.i.d. coefficients above
# model none of that).  The coefficient fields Cq, Ck [F, Hh, Ww, R] are white noise passed
# through a periodic Gaussian low-pass of width `sigma` voxels along every grid axis and
# rescaled to unit variance; everything else is the recipe of head_tensors.  The correlation
# of two coefficient vectors at grid offset D is exp(-|D|^2 / (4 sigma^2)).
# ---------------------------------------------------------------------------------------

def _smooth_field(white: np.ndarray, sigma: float) -> np.ndarray:
    """white [F, Hh, Ww, R] -> same shape, Gaussian low-pass over the three grid axes (periodic), unit variance."""
    f = np.fft.rfftn(white, axes=(0, 1, 2))
    for ax, n in enumerate(white.shape[:3]):
        freq = np.fft.rfftfreq(n) if ax == 2 else np.fft.fftfreq(n)
        gain = np.exp(-2.0 * (np.pi * freq * sigma) ** 2)
        shape = [1, 1, 1, 1]
        shape[ax] = gain.shape[0]
        f *= gain.reshape(shape)
    out = np.fft.irfftn(f, s=white.shape[:3], axes=(0, 1, 2))
    return out / out.std()


def head_tensors_smooth(cfg: WorkloadConfig, head: int, seed: int = 0, sigma: float = 5.0,
                        names=("Q", "K", "V", "dO")) -> dict:
    """As head_tensors, with the Q / K coefficient fields smooth over cfg.grid (V, dO unchanged)."""
    out = {}
    L, d, R = cfg.L, cfg.d, cfg.basis_rank
    G = basis(cfg, seed)
    for name in names:
        rng = _rng(seed, cfg.index, name, head, extra=1)
        if name in ("Q", "K"):
            coef = _smooth_field(rng.standard_normal(tuple(cfg.grid) + (R,)), sigma).reshape(L, R)
            noise = rng.standard_normal((L, d), dtype=np.float32)
            x = (coef @ G).astype(np.float32) + np.float32(0.1) * noise
        else:
            x = rng.standard_normal((L, d), dtype=np.float32)
        out[name] = round_to_dtype(x, cfg.dtype)
    return out
