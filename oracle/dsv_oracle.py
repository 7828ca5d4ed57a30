"""ctypes front end of the C oracle (oracle/dsv_oracle.c).  Test infrastructure only.

Marshals numpy arrays into the plain C routines; all arithmetic lives in the C file.
Tensors are float32 arrays holding storage-dtype-rounded values; results come back as
float64 (indices as int32).  Nothing here is imported by the product package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dsv_oracle.c")
_LIB = os.path.join(_HERE, "libdsv_oracle.so")

DTYPES = {"f32": 0, "bf16": 1}

__all__ = ["build", "lib", "round_value", "project", "scores", "topk_from_scores", "lowrank_topk",
           "sparse_fwd", "sparse_bwd", "sparse_bwd_rows", "sparse_bwd_dq_rows", "sparse_bwd_dkdv_key",
           "dense_fwd", "dense_bwd", "max_threads", "DTYPES", "group_member", "group_centre", "group_tokens",
           "lowrank_topk_grouped", "group_expand_idx", "group_overlap", "sparse_fwd_grouped", "sparse_bwd_grouped",
           "predictor_loss", "profile_sparsity", "ema"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction) and return the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.dsv_oracle_round.restype = ctypes.c_double
        L.dsv_oracle_round.argtypes = [ctypes.c_double, ctypes.c_int]
        L.dsv_oracle_max_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p) if a is not None else None


_i64 = ctypes.c_int64
_int = ctypes.c_int
_dbl = ctypes.c_double


def max_threads() -> int:
    return int(lib().dsv_oracle_max_threads())


def round_value(x: float, dtype: str) -> float:
    return float(lib().dsv_oracle_round(float(x), DTYPES[dtype]))


def project(X, W, dtype: str) -> np.ndarray:
    """rnd(X W): X [n, d], W [d, r] -> [n, r] float32 holding dtype-rounded values."""
    X, W = _f32(X), _f32(W)
    n, d = X.shape
    r = W.shape[1]
    assert W.shape[0] == d
    out = np.empty((n, r), dtype=np.float32)
    lib().dsv_oracle_project(_p(X), _p(W), _i64(n), _int(d), _int(r), _int(DTYPES[dtype]), _p(out))
    return out


def scores(Qlr, Klr) -> np.ndarray:
    """Qlr [nq, r], Klr [L, r] -> S [nq, L] float64."""
    Qlr, Klr = _f32(Qlr), _f32(Klr)
    nq, r = Qlr.shape
    L = Klr.shape[0]
    assert Klr.shape[1] == r
    S = np.empty((nq, L), dtype=np.float64)
    lib().dsv_oracle_scores(_p(Qlr), _p(Klr), _i64(nq), _i64(L), _int(r), _p(S))
    return S


def topk_from_scores(S, k: int) -> np.ndarray:
    """S [nq, L] -> idx [nq, k] int32, ascending; larger score wins, ties to the lower index."""
    S = _f64(S)
    nq, L = S.shape
    assert 1 <= k <= L
    idx = np.empty((nq, k), dtype=np.int32)
    lib().dsv_oracle_topk_from_scores(_p(S), _i64(nq), _i64(L), _i64(k), _p(idx))
    return idx


def lowrank_topk(Q_rows, K, Wq, Wk, k: int, dtype: str, return_intermediates: bool = False):
    """Stage 1 for the given query rows of one head.  Q_rows [nq, d], K [L, d], Wq, Wk [d, r]."""
    Q_rows, K, Wq, Wk = _f32(Q_rows), _f32(K), _f32(Wq), _f32(Wk)
    nq, d = Q_rows.shape
    L = K.shape[0]
    r = Wq.shape[1]
    assert K.shape[1] == d and Wq.shape == (d, r) and Wk.shape == (d, r) and 1 <= k <= L
    idx = np.empty((nq, k), dtype=np.int32)
    Qlr = np.empty((nq, r), dtype=np.float32) if return_intermediates else None
    Klr = np.empty((L, r), dtype=np.float32) if return_intermediates else None
    S = np.empty((nq, L), dtype=np.float64) if return_intermediates else None
    lib().dsv_oracle_lowrank_topk(_p(Q_rows), _p(K), _p(Wq), _p(Wk), _i64(nq), _i64(L), _int(d), _int(r),
                                  _i64(k), _int(DTYPES[dtype]), _p(idx), _p(Qlr), _p(Klr), _p(S))
    if return_intermediates:
        return idx, Qlr, Klr, S
    return idx


def sparse_fwd(Q_rows, K, V, idx_rows, scale: float, return_p: bool = False):
    """Sparse attention forward for the given query rows -> (O [nq, d], lse [nq][, P [nq, k]])."""
    Q_rows, K, V, idx_rows = _f32(Q_rows), _f32(K), _f32(V), _i32(idx_rows)
    nq, d = Q_rows.shape
    L = K.shape[0]
    k = idx_rows.shape[1]
    assert idx_rows.shape[0] == nq and K.shape == V.shape == (L, d)
    assert idx_rows.min() >= 0 and idx_rows.max() < L
    O = np.empty((nq, d), dtype=np.float64)
    lse = np.empty(nq, dtype=np.float64)
    P = np.empty((nq, k), dtype=np.float64) if return_p else None
    lib().dsv_oracle_sparse_fwd(_p(Q_rows), _p(K), _p(V), _p(idx_rows), _i64(nq), _i64(L), _int(d), _i64(k),
                                _dbl(scale), _p(O), _p(lse), _p(P))
    return (O, lse, P) if return_p else (O, lse)


def sparse_bwd(Q, K, V, idx, dO, scale: float):
    """Whole-head backward (runs the oracle forward first) -> (dQ, dK, dV) float64 [L, d]."""
    Q, K, V, dO, idx = _f32(Q), _f32(K), _f32(V), _f32(dO), _i32(idx)
    L, d = Q.shape
    k = idx.shape[1]
    assert idx.shape[0] == L and K.shape == V.shape == dO.shape == (L, d)
    O, lse = sparse_fwd(Q, K, V, idx, scale)
    dQ = np.empty((L, d)); dK = np.empty((L, d)); dV = np.empty((L, d))
    lib().dsv_oracle_sparse_bwd(_p(Q), _p(K), _p(V), _p(idx), _p(O), _p(lse), _p(dO), _i64(L), _int(d),
                                _i64(k), _dbl(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def sparse_bwd_rows(Q_rows, K, V, idx_rows, dO_rows, scale: float):
    """Backward of the given query rows: (dQ [nq, d], dK [L, d], dV [L, d]) where dK, dV hold only
    these rows' contributions (all of a head's rows give the whole-head gradients)."""
    Q_rows, K, V, dO_rows, idx_rows = _f32(Q_rows), _f32(K), _f32(V), _f32(dO_rows), _i32(idx_rows)
    nq, d = Q_rows.shape
    L = K.shape[0]
    k = idx_rows.shape[1]
    O, lse = sparse_fwd(Q_rows, K, V, idx_rows, scale)
    dQ = np.empty((nq, d)); dK = np.zeros((L, d)); dV = np.zeros((L, d))
    lib().dsv_oracle_sparse_bwd_rows(_p(Q_rows), _p(K), _p(V), _p(idx_rows), _p(O), _p(lse), _p(dO_rows),
                                     _i64(nq), _int(d), _i64(k), _dbl(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


def sparse_bwd_dq_rows(Q_rows, K, V, idx_rows, dO_rows, scale: float):
    """dQ of the given query rows only -> [nq, d] float64."""
    Q_rows, K, V, dO_rows, idx_rows = _f32(Q_rows), _f32(K), _f32(V), _f32(dO_rows), _i32(idx_rows)
    nq, d = Q_rows.shape
    k = idx_rows.shape[1]
    O, lse = sparse_fwd(Q_rows, K, V, idx_rows, scale)
    dQ = np.empty((nq, d))
    lib().dsv_oracle_sparse_bwd_dq_rows(_p(Q_rows), _p(K), _p(V), _p(idx_rows), _p(O), _p(lse), _p(dO_rows),
                                        _i64(nq), _int(d), _i64(k), _dbl(scale), _p(dQ))
    return dQ


def sparse_bwd_dkdv_key(j: int, Q_sel, dO_sel, idx_sel, K, V, scale: float):
    """dK_j, dV_j of one key from the rows (Q_sel, dO_sel, idx_sel) of every query that selected it."""
    Q_sel, dO_sel, idx_sel, K, V = _f32(Q_sel), _f32(dO_sel), _i32(idx_sel), _f32(K), _f32(V)
    n, d = Q_sel.shape
    k = idx_sel.shape[1] if n else 1
    dKj = np.zeros(d); dVj = np.zeros(d)
    if n == 0:
        return dKj, dVj
    assert (idx_sel == j).sum(axis=1).min() == 1
    O, lse = sparse_fwd(Q_sel, K, V, idx_sel, scale)
    lib().dsv_oracle_sparse_bwd_dkdv_key(ctypes.c_int32(j), _p(Q_sel), _p(dO_sel), _p(O), _p(lse), _p(idx_sel),
                                         _i64(n), _p(K), _p(V), _int(d), _i64(k), _dbl(scale), _p(dKj), _p(dVj))
    return dKj, dVj


def dense_fwd(Q, K, V, scale: float, return_p: bool = False):
    Q, K, V = _f32(Q), _f32(K), _f32(V)
    L, d = Q.shape
    O = np.empty((L, d)); lse = np.empty(L)
    P = np.empty((L, L)) if return_p else None
    lib().dsv_oracle_dense_fwd(_p(Q), _p(K), _p(V), _i64(L), _int(d), _dbl(scale), _p(O), _p(lse), _p(P))
    return (O, lse, P) if return_p else (O, lse)


def dense_bwd(Q, K, V, dO, scale: float):
    Q, K, V, dO = _f32(Q), _f32(K), _f32(V), _f32(dO)
    L, d = Q.shape
    dQ = np.empty((L, d)); dK = np.empty((L, d)); dV = np.empty((L, d))
    lib().dsv_oracle_dense_bwd(_p(Q), _p(K), _p(V), _p(dO), _i64(L), _int(d), _dbl(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


# ---- query grouping ---------------------------------------------------------------------------
def group_member(g: int, m: int, grid, cube) -> int:
    """Token index of member m of group g on a (frames, height, width) grid tiled by `cube`."""
    L = lib()
    L.dsv_oracle_group_member.restype = ctypes.c_int64
    return int(L.dsv_oracle_group_member(_i64(g), _int(m), *[_int(x) for x in grid], *[_int(x) for x in cube]))


def group_centre(cube) -> int:
    return int(lib().dsv_oracle_group_centre(*[_int(x) for x in cube]))


def group_tokens(grid, cube) -> np.ndarray:
    """int64 [n_groups, G]: token index of every member of every group (from the C routine)."""
    Ltok = grid[0] * grid[1] * grid[2]
    G = cube[0] * cube[1] * cube[2]
    return np.array([[group_member(g, m, grid, cube) for m in range(G)] for g in range(Ltok // G)], dtype=np.int64)


def lowrank_topk_grouped(Q, K, Wq, Wk, grid, cube, k: int, dtype: str) -> np.ndarray:
    """idx_g [n_groups, k]: per group, the centre query's k best keys."""
    Q, K, Wq, Wk = _f32(Q), _f32(K), _f32(Wq), _f32(Wk)
    Ltok, d = Q.shape
    r = Wq.shape[1]
    G = cube[0] * cube[1] * cube[2]
    assert Ltok == grid[0] * grid[1] * grid[2] and all(a % b == 0 for a, b in zip(grid, cube))
    idx_g = np.empty((Ltok // G, k), dtype=np.int32)
    lib().dsv_oracle_lowrank_topk_grouped(_p(Q), _p(K), _p(Wq), _p(Wk), *[_int(x) for x in grid], *[_int(x) for x in cube],
                                          _int(d), _int(r), _i64(k), _int(DTYPES[dtype]), _p(idx_g))
    return idx_g


def group_expand_idx(idx_g, grid, cube) -> np.ndarray:
    idx_g = _i32(idx_g)
    Ltok = grid[0] * grid[1] * grid[2]
    k = idx_g.shape[1]
    idx = np.empty((Ltok, k), dtype=np.int32)
    lib().dsv_oracle_group_expand_idx(_p(idx_g), *[_int(x) for x in grid], *[_int(x) for x in cube], _i64(k), _p(idx))
    return idx


def sparse_fwd_grouped(Q, K, V, idx_g, grid, cube, scale: float):
    Q, K, V, idx_g = _f32(Q), _f32(K), _f32(V), _i32(idx_g)
    Ltok, d = Q.shape
    k = idx_g.shape[1]
    O = np.empty((Ltok, d)); lse = np.empty(Ltok)
    lib().dsv_oracle_sparse_fwd_grouped(_p(Q), _p(K), _p(V), _p(idx_g), *[_int(x) for x in grid], *[_int(x) for x in cube],
                                        _int(d), _i64(k), _dbl(scale), _p(O), _p(lse))
    return O, lse


def sparse_bwd_grouped(Q, K, V, idx_g, dO, grid, cube, scale: float):
    Q, K, V, dO, idx_g = _f32(Q), _f32(K), _f32(V), _f32(dO), _i32(idx_g)
    Ltok, d = Q.shape
    k = idx_g.shape[1]
    dQ = np.empty((Ltok, d)); dK = np.empty((Ltok, d)); dV = np.empty((Ltok, d))
    lib().dsv_oracle_sparse_bwd_grouped(_p(Q), _p(K), _p(V), _p(idx_g), _p(dO), *[_int(x) for x in grid],
                                        *[_int(x) for x in cube], _int(d), _i64(k), _dbl(scale), _p(dQ), _p(dK), _p(dV))
    return dQ, dK, dV


# ---- predictor side ---------------------------------------------------------------------------
def group_overlap(idx, grid, cube) -> float:
    """Mean share of a query's own selection (idx [L, k], per-query rows) that its group centre's row also holds."""
    idx = _i32(idx)
    L, k = idx.shape
    F, Hh, Ww = grid
    gf, gh, gw = cube
    fn = lib().dsv_oracle_group_overlap
    fn.restype = ctypes.c_int64
    count = fn(_p(idx), _int(F), _int(Hh), _int(Ww), _int(gf), _int(gh), _int(gw), _i64(k))
    if count < 0:
        raise ValueError("the cube does not tile the grid")
    return count / (L * k)


def predictor_loss(Q_rows, K, Wq, Wk):
    """0.95 CosLoss + 0.05 NormLoss of the low-rank scores of the given query rows against the true ones, and its
    gradients: ((loss, cos, norm), dWq [d, r], dWk [d, r])."""
    Q_rows, K, Wq, Wk = _f32(Q_rows), _f32(K), _f32(Wq), _f32(Wk)
    n, d = Q_rows.shape
    L = K.shape[0]
    r = Wq.shape[1]
    parts = np.empty(3); dWq = np.empty((d, r)); dWk = np.empty((d, r))
    lib().dsv_oracle_predictor_loss(_p(Q_rows), _p(K), _p(Wq), _p(Wk), _i64(n), _i64(L), _int(d), _int(r), _p(parts),
                                    _p(dWq), _p(dWk))
    return tuple(float(x) for x in parts), dWq, dWk


def profile_sparsity(Q_rows, K, scale: float, mass: float = 0.9):
    """(head sparsity on the sampled rows, counts [n] of critical keys per row)."""
    Q_rows, K = _f32(Q_rows), _f32(K)
    n, d = Q_rows.shape
    L = K.shape[0]
    counts = np.empty(n, dtype=np.int64)
    L_ = lib()
    L_.dsv_oracle_profile_sparsity.restype = ctypes.c_double
    s = L_.dsv_oracle_profile_sparsity(_p(Q_rows), _p(K), _i64(n), _i64(L), _int(d), _dbl(scale), _dbl(mass), _p(counts))
    return float(s), counts


def ema(prev: float, sample: float, alpha: float) -> float:
    L_ = lib()
    L_.dsv_oracle_ema.restype = ctypes.c_double
    return float(L_.dsv_oracle_ema(_dbl(prev), _dbl(sample), _dbl(alpha)))
