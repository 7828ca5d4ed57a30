"""Pins of the CPU oracle's stage 1 (projection, scores, selection) against things other than
itself: hand-derived rounding cases, exact rational arithmetic, numpy's GEMM, numpy's lexsort,
a pure-Python brute-force sort, and closed-form special cases."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
import workloads as wl


# ----------------------------------------------------------------------------- rounding
def test_round_bf16_hand_cases():
    r = lambda x: oracle.round_value(x, "bf16")
    assert r(1.0) == 1.0
    assert r(1 + 2**-8) == 1.0                      # tie -> even (down)
    assert r(1 + 3 * 2**-8) == 1 + 2**-6            # tie -> even (up)
    assert r(1 + 2**-8 + 2**-40) == 1 + 2**-7       # just above the tie, straight from double
    assert r(-(1 + 2**-8 + 2**-40)) == -(1 + 2**-7)
    assert r(255.5) == 256.0 and r(254.5) == 254.0 and r(257.0) == 256.0 and r(259.0) == 260.0
    assert r(2.0**-133) == 2.0**-133                # smallest bf16 subnormal survives
    assert r(2.0**-134) == 0.0                      # half of it ties to even (zero)
    assert r(0.0) == 0.0


def test_round_f32_hand_cases():
    r = lambda x: oracle.round_value(x, "f32")
    assert r(1 + 2**-24) == 1.0
    assert r(1 + 2**-24 + 2**-50) == 1 + 2**-23
    assert r(1 + 3 * 2**-24) == 1 + 2**-22
    assert r(0.1) == float(np.float32(0.1))


def test_round_matches_library_conversion():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal(4000) * np.exp(rng.uniform(-20, 20, 4000))).astype(np.float32)
    lib_bf16 = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    mine = np.array([oracle.round_value(float(v), "bf16") for v in x], dtype=np.float32)
    assert np.array_equal(lib_bf16, mine)
    xd = rng.standard_normal(2000) * np.exp(rng.uniform(-20, 20, 2000))
    assert np.array_equal(xd.astype(np.float32),
                          np.array([oracle.round_value(float(v), "f32") for v in xd], dtype=np.float32))


def test_round_bf16_is_nearest_in_exact_arithmetic():
    rng = np.random.default_rng(2)
    for v in rng.standard_normal(300) * 7.3:
        got = Fraction(oracle.round_value(float(v), "bf16"))
        e = int(np.floor(np.log2(abs(v))))
        ulp = Fraction(2) ** (e - 7)
        assert abs(got - Fraction(float(v))) <= ulp / 2
        assert (got / ulp).denominator == 1            # representable with 8 significant bits


# ----------------------------------------------------------------------------- projection
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_project_is_a_rounded_gemm(dtype):
    rng = np.random.default_rng(3)
    n, d, r = 37, 48, 16
    X = wl.round_to_dtype(rng.standard_normal((n, d)), dtype)
    W = wl.round_to_dtype(rng.standard_normal((d, r)) / np.sqrt(d), dtype)
    got = oracle.project(X, W, dtype)
    exact = X.astype(np.float64) @ W.astype(np.float64)
    assert got.shape == (n, r)
    prec = 8 if dtype == "bf16" else 24
    ulp = 2.0 ** (np.floor(np.log2(np.abs(exact))) - (prec - 1))
    assert np.all(np.abs(got - exact) <= 0.5 * ulp * (1 + 1e-9))
    if dtype == "bf16":
        assert not np.any(got.view(np.uint32) & 0xFFFF)
    # a transposed or mis-strided operand cannot pass: compare one entry against a hand sum
    i, t = 5, 11
    hand = sum(float(X[i, c]) * float(W[c, t]) for c in range(d))
    assert got[i, t] == np.float32(oracle.round_value(hand, dtype))


def test_project_integer_inputs_exact():
    Q, K, Wq, Wk = wl.ternary_head_tensors(64, 128, 16, seed=4)
    got = oracle.project(Q, Wq, "bf16")
    assert np.array_equal(got, (Q.astype(np.int64) @ Wq.astype(np.int64)).astype(np.float32))


# ----------------------------------------------------------------------------- scores
def test_scores_is_qlr_klr_transpose():
    rng = np.random.default_rng(5)
    Qlr = wl.round_to_dtype(rng.standard_normal((9, 16)), "bf16")
    Klr = wl.round_to_dtype(rng.standard_normal((21, 16)), "bf16")
    S = oracle.scores(Qlr, Klr)
    assert S.shape == (9, 21)
    # bf16 x bf16 products of <= 32 terms are exact in double: equality, not closeness
    exact = np.array([[sum(Fraction(float(a)) * Fraction(float(b)) for a, b in zip(q, k)) for k in Klr] for q in Qlr])
    assert all(Fraction(float(S[i, j])) == exact[i, j] for i in range(9) for j in range(21))
    assert np.allclose(S, Qlr.astype(np.float64) @ Klr.astype(np.float64).T, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- selection
def _brute_topk(S, k):
    out = []
    for row in S:
        order = sorted(range(len(row)), key=lambda j: (-row[j], j))
        out.append(sorted(order[:k]))
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("L,k", [(1, 1), (7, 3), (64, 64), (257, 31), (300, 299)])
def test_topk_matches_brute_force_with_ties(L, k):
    rng = np.random.default_rng(6 + L)
    S = rng.integers(-3, 4, size=(11, L)).astype(np.float64)      # few distinct values: many ties
    assert np.array_equal(oracle.topk_from_scores(S, k), _brute_topk(S, k))
    S = rng.standard_normal((11, L))
    assert np.array_equal(oracle.topk_from_scores(S, k), _brute_topk(S, k))


def test_topk_matches_lexsort():
    rng = np.random.default_rng(7)
    S = np.round(rng.standard_normal((20, 500)) * 4) / 4
    k = 77
    ref = np.stack([np.sort(np.lexsort((np.arange(500), -row))[:k]) for row in S]).astype(np.int32)
    assert np.array_equal(oracle.topk_from_scores(S, k), ref)


def test_topk_special_cases():
    L = 50
    assert np.array_equal(oracle.topk_from_scores(np.zeros((3, L)), 9), np.tile(np.arange(9), (3, 1)))
    S = np.random.default_rng(8).standard_normal((4, L))
    assert np.array_equal(oracle.topk_from_scores(S, L), np.tile(np.arange(L), (4, 1)))
    assert np.array_equal(oracle.topk_from_scores(S, 1)[:, 0], S.argmax(axis=1))
    # -0.0 and +0.0 tie; the lower index wins
    S0 = np.full((1, 6), -1.0); S0[0, 4] = 0.0; S0[0, 2] = -0.0
    assert oracle.topk_from_scores(S0, 1)[0, 0] == 2
    # largest-first, not smallest-first
    S1 = np.arange(10, dtype=np.float64)[None, :]
    assert np.array_equal(oracle.topk_from_scores(S1, 3)[0], [7, 8, 9])


def test_lowrank_topk_with_identity_predictor_is_exact_topk_of_qkt():
    rng = np.random.default_rng(9)
    L, d, k = 96, 16, 10
    Q = rng.integers(-4, 5, size=(L, d)).astype(np.float32)
    K = rng.integers(-4, 5, size=(L, d)).astype(np.float32)
    I = np.eye(d, dtype=np.float32)
    idx = oracle.lowrank_topk(Q, K, I, I, k, "bf16")
    S = Q.astype(np.int64) @ K.astype(np.int64).T
    ref = np.stack([np.sort(np.argsort(-row, kind="stable")[:k]) for row in S]).astype(np.int32)
    assert np.array_equal(idx, ref)


def test_lowrank_topk_composes_its_parts_and_uses_wq_for_q_wk_for_k():
    cfg = wl.get_config(0)
    t = wl.head_tensors(cfg, 1, names=("Q", "K"))
    Wq, Wk = wl.predictor_weights(cfg, 1)
    rows = np.array([0, 5, 1023])
    idx, Qlr, Klr, S = oracle.lowrank_topk(t["Q"][rows], t["K"], Wq, Wk, cfg.k, cfg.dtype, return_intermediates=True)
    Qlr_np = (t["Q"][rows].astype(np.float64) @ Wq.astype(np.float64)).astype(np.float32)
    Klr_np = (t["K"].astype(np.float64) @ Wk.astype(np.float64)).astype(np.float32)
    assert np.array_equal(Qlr, Qlr_np) and np.array_equal(Klr, Klr_np)
    S_np = Qlr_np.astype(np.float64) @ Klr_np.astype(np.float64).T
    assert np.allclose(S, S_np, rtol=0, atol=1e-12)
    assert np.array_equal(idx, _brute_topk(S, cfg.k))
    assert idx.shape == (3, cfg.k) and np.all(np.diff(idx, axis=1) > 0)
