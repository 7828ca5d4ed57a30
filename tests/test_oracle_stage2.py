"""Pins of the CPU oracle's stage 2 (sparse attention forward / backward) against library
routines (torch scaled_dot_product_attention and autograd in float64, with the unselected keys
masked out), closed forms, identities and central finite differences."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import workloads as wl


def _inputs(L, d, seed, dtype="bf16"):
    rng = np.random.default_rng(seed)
    mk = lambda s=1.0: wl.round_to_dtype(rng.standard_normal((L, d)) * s, dtype)
    return mk(), mk(), mk(), mk()


def _torch_masked(Q, K, V, idx, scale, dO=None):
    """softmax(scale Q K^T + mask) V in float64 by the library, mask = -inf off the index set."""
    L = K.shape[0]
    q = torch.tensor(Q, dtype=torch.float64, requires_grad=True)
    k = torch.tensor(K, dtype=torch.float64, requires_grad=True)
    v = torch.tensor(V, dtype=torch.float64, requires_grad=True)
    mask = torch.zeros((Q.shape[0], L), dtype=torch.bool)
    mask.scatter_(1, torch.tensor(idx, dtype=torch.int64), True)
    o = F.scaled_dot_product_attention(q[None, None], k[None, None], v[None, None],
                                       attn_mask=mask[None, None], scale=scale)[0, 0]
    if dO is None:
        return o.detach().numpy()
    o.backward(torch.tensor(dO, dtype=torch.float64))
    return o.detach().numpy(), q.grad.numpy(), k.grad.numpy(), v.grad.numpy()


# ----------------------------------------------------------------------------- forward
def test_dense_fwd_is_library_attention():
    Q, K, V, _ = _inputs(33, 16, 1)
    scale = 0.31
    O, lse, P = oracle.dense_fwd(Q, K, V, scale, return_p=True)
    ref = F.scaled_dot_product_attention(*(torch.tensor(x, dtype=torch.float64)[None] for x in (Q, K, V)), scale=scale)[0]
    assert np.allclose(O, ref.numpy(), rtol=0, atol=1e-13)
    S = scale * Q.astype(np.float64) @ K.astype(np.float64).T
    assert np.allclose(lse, torch.logsumexp(torch.tensor(S), dim=1).numpy(), rtol=0, atol=1e-13)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13)


@pytest.mark.parametrize("L,d,k", [(40, 8, 40), (40, 8, 7), (129, 64, 33), (64, 128, 1)])
def test_sparse_fwd_is_masked_library_attention(L, d, k):
    Q, K, V, _ = _inputs(L, d, 2 + k)
    idx = wl.random_subset_idx(L, k, L, seed=3)
    scale = 1.0 / np.sqrt(d)
    O, lse, P = oracle.sparse_fwd(Q, K, V, idx, scale, return_p=True)
    assert np.allclose(O, _torch_masked(Q, K, V, idx, scale), rtol=0, atol=1e-13)
    S = scale * Q.astype(np.float64) @ K.astype(np.float64).T
    S_sel = np.take_along_axis(S, idx.astype(np.int64), axis=1)
    assert np.allclose(lse, torch.logsumexp(torch.tensor(S_sel), dim=1).numpy(), rtol=0, atol=1e-13)
    assert np.allclose(P.sum(axis=1), 1.0, atol=1e-13)
    assert np.allclose(np.exp(lse), np.exp(S_sel).sum(axis=1), rtol=1e-12)


def test_sparse_fwd_at_k_equals_L_is_dense():
    L, d = 48, 16
    Q, K, V, _ = _inputs(L, d, 5)
    Od, lsed = oracle.dense_fwd(Q, K, V, 0.2)
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    Os, lses = oracle.sparse_fwd(Q, K, V, idx, 0.2)
    assert np.allclose(Os, Od, rtol=0, atol=1e-14) and np.allclose(lses, lsed, rtol=0, atol=1e-14)


def test_sparse_fwd_closed_forms():
    L, d, k = 30, 8, 6
    Q, K, V, _ = _inputs(L, d, 6)
    idx = wl.random_subset_idx(L, k, L, seed=7)
    # k = 1: the output is the selected value row, lse is the single score
    idx1 = idx[:, :1].copy()
    O, lse = oracle.sparse_fwd(Q, K, V, idx1, 0.5)
    assert np.array_equal(O, V[idx1[:, 0]].astype(np.float64))
    s = 0.5 * np.einsum("ic,ic->i", Q.astype(np.float64), K[idx1[:, 0]].astype(np.float64))
    assert np.allclose(lse, s, rtol=0, atol=1e-14)
    # Q = 0: uniform weights over the selected rows, lse = log k
    O, lse = oracle.sparse_fwd(np.zeros_like(Q), K, V, idx, 0.5)
    assert np.allclose(O, V[idx].astype(np.float64).mean(axis=1), rtol=0, atol=1e-14)
    assert np.allclose(lse, np.log(k), rtol=0, atol=1e-14)
    # the order of an index row does not matter
    Oa, lsea = oracle.sparse_fwd(Q, K, V, idx, 0.5)
    perm = np.random.default_rng(8).permuted(idx, axis=1)
    Ob, lseb = oracle.sparse_fwd(Q, K, V, perm, 0.5)
    assert np.allclose(Oa, Ob, rtol=0, atol=1e-14) and np.allclose(lsea, lseb, rtol=0, atol=1e-14)
    # the scale multiplies the logits (not the output): doubling Q equals doubling the scale
    Oc, lsec = oracle.sparse_fwd(2 * Q, K, V, idx, 0.25)
    assert np.allclose(Oa, Oc, rtol=0, atol=1e-14) and np.allclose(lsea, lsec, rtol=0, atol=1e-14)


def test_sparse_fwd_on_row_subset_uses_the_rows_it_is_given():
    L, d, k = 50, 16, 9
    Q, K, V, _ = _inputs(L, d, 9)
    idx = wl.random_subset_idx(L, k, L, seed=10)
    O, lse = oracle.sparse_fwd(Q, K, V, idx, 0.3)
    rows = np.array([3, 17, 49])
    Or, lser = oracle.sparse_fwd(Q[rows], K, V, idx[rows], 0.3)
    assert np.array_equal(Or, O[rows]) and np.array_equal(lser, lse[rows])


# ----------------------------------------------------------------------------- backward
@pytest.mark.parametrize("L,d,k", [(24, 8, 24), (40, 16, 9), (65, 64, 17)])
def test_sparse_bwd_is_library_autograd_of_masked_attention(L, d, k):
    Q, K, V, dO = _inputs(L, d, 11 + k)
    idx = wl.random_subset_idx(L, k, L, seed=12)
    scale = 1.7 / np.sqrt(d)
    dQ, dK, dV = oracle.sparse_bwd(Q, K, V, idx, dO, scale)
    _, gq, gk, gv = _torch_masked(Q, K, V, idx, scale, dO)
    assert np.allclose(dQ, gq, rtol=0, atol=1e-12)
    assert np.allclose(dK, gk, rtol=0, atol=1e-12)
    assert np.allclose(dV, gv, rtol=0, atol=1e-12)


def test_dense_bwd_is_library_autograd_and_the_k_equals_L_limit():
    L, d = 20, 8
    Q, K, V, dO = _inputs(L, d, 13)
    scale = 0.4
    dQ, dK, dV = oracle.dense_bwd(Q, K, V, dO, scale)
    idx = np.tile(np.arange(L, dtype=np.int32), (L, 1))
    _, gq, gk, gv = _torch_masked(Q, K, V, idx, scale, dO)
    for a, b in ((dQ, gq), (dK, gk), (dV, gv)):
        assert np.allclose(a, b, rtol=0, atol=1e-12)
    sQ, sK, sV = oracle.sparse_bwd(Q, K, V, idx, dO, scale)
    for a, b in ((dQ, sQ), (dK, sK), (dV, sV)):
        assert np.allclose(a, b, rtol=0, atol=1e-13)


def test_sparse_bwd_finite_differences():
    L, d, k = 12, 4, 5
    rng = np.random.default_rng(14)
    Q, K, V, dO = (rng.standard_normal((L, d)).astype(np.float32) for _ in range(4))
    idx = wl.random_subset_idx(L, k, L, seed=15)
    scale = 0.6
    dQ, dK, dV = oracle.sparse_bwd(Q, K, V, idx, dO, scale)

    def loss(q, kk, v):
        O, _ = oracle.sparse_fwd(q, kk, v, idx, scale)
        return float((O * dO.astype(np.float64)).sum())

    h = 2.0 ** -10            # exactly representable steps keep the float32 containers exact
    for name, g in (("Q", dQ), ("K", dK), ("V", dV)):
        for (i, c) in [(0, 0), (3, 2), (11, 3), (7, 1)]:
            args_p = [Q.copy(), K.copy(), V.copy()]
            args_m = [Q.copy(), K.copy(), V.copy()]
            t = "QKV".index(name)
            base = np.float32(np.round(args_p[t][i, c] * 1024) / 1024)   # put the point on the grid
            for a in (args_p, args_m):
                a[t][i, c] = base
            if t == 0:
                Q2 = args_p[0].copy(); ref = oracle.sparse_bwd(Q2, K, V, idx, dO, scale)[0][i, c]
            elif t == 1:
                K2 = args_p[1].copy(); ref = oracle.sparse_bwd(Q, K2, V, idx, dO, scale)[1][i, c]
            else:
                V2 = args_p[2].copy(); ref = oracle.sparse_bwd(Q, K, V2, idx, dO, scale)[2][i, c]
            args_p[t][i, c] = base + np.float32(h)
            args_m[t][i, c] = base - np.float32(h)
            fd = (loss(*args_p) - loss(*args_m)) / (2 * h)
            assert abs(fd - ref) <= 1e-5 * max(1.0, abs(ref)), (name, i, c, fd, ref)


def test_sparse_bwd_identities():
    L, d, k = 60, 16, 7
    Q, K, V, dO = _inputs(L, d, 16)
    idx = wl.random_subset_idx(L, k, L, seed=17)
    dQ, dK, dV = oracle.sparse_bwd(Q, K, V, idx, dO, 0.25)
    # rows of P sum to one  =>  sum_j dV_j = sum_i dO_i
    assert np.allclose(dV.sum(axis=0), dO.astype(np.float64).sum(axis=0), rtol=0, atol=1e-12)
    # keys nobody selected get exact zeros
    unselected = np.setdiff1d(np.arange(L), np.unique(idx))
    forced = wl.random_subset_idx(L - 5, k, L, seed=18)        # keys L-5..L-1 never selected
    _, dK2, dV2 = oracle.sparse_bwd(Q, K, V, forced, dO, 0.25)
    assert np.all(dK2[L - 5:] == 0.0) and np.all(dV2[L - 5:] == 0.0)
    assert np.all(dK[unselected] == 0.0) and np.all(dV[unselected] == 0.0)
    # sum_j dS_ij = 0 for every row: adding one common vector to every key (a constant shift of
    # each row's logits, which softmax ignores) leaves dQ unchanged
    shift = np.float32(0.5) * np.ones((1, d), dtype=np.float32)
    dQs, _, _ = oracle.sparse_bwd(Q, K + shift, V, idx, dO, 0.25)
    assert np.allclose(dQs, dQ, rtol=0, atol=1e-12)


def test_row_and_key_sampled_backward_agree_with_the_whole_head():
    L, d, k = 80, 32, 11
    Q, K, V, dO = _inputs(L, d, 19)
    idx = wl.random_subset_idx(L, k, L, seed=20)
    dQ, dK, dV = oracle.sparse_bwd(Q, K, V, idx, dO, 0.2)
    rows = np.array([0, 41, 79])
    assert np.allclose(oracle.sparse_bwd_dq_rows(Q[rows], K, V, idx[rows], dO[rows], 0.2), dQ[rows], rtol=0, atol=1e-14)
    # two halves of the rows: their dK / dV contributions add up to the whole head's
    a, b = np.arange(0, 37), np.arange(37, L)
    dQa, dKa, dVa = oracle.sparse_bwd_rows(Q[a], K, V, idx[a], dO[a], 0.2)
    dQb, dKb, dVb = oracle.sparse_bwd_rows(Q[b], K, V, idx[b], dO[b], 0.2)
    assert np.allclose(np.concatenate([dQa, dQb]), dQ, rtol=0, atol=1e-14)
    assert np.allclose(dKa + dKb, dK, rtol=0, atol=1e-13) and np.allclose(dVa + dVb, dV, rtol=0, atol=1e-13)
    for j in (0, 7, 79):
        sel = np.nonzero((idx == j).any(axis=1))[0]
        dKj, dVj = oracle.sparse_bwd_dkdv_key(j, Q[sel], dO[sel], idx[sel], K, V, 0.2)
        assert np.allclose(dKj, dK[j], rtol=0, atol=1e-13) and np.allclose(dVj, dV[j], rtol=0, atol=1e-13)


# ----------------------------------------------------------------------------- the regime
def test_generator_puts_about_90_percent_of_the_mass_on_the_top_6_percent():
    """Paper, Sec. "Empirical Observations": the top ~10 % of keys hold ~90 % of a query's
    attention.  With the config-1 recipe (d=128, basis rank 64, scale 2/sqrt(d)) the logits are
    ~N(0, 2.83^2) and the top 6.25 % of keys hold Phi(2.83 - 1.53) ~ 0.90 of the softmax mass."""
    cfg = wl.get_config(1)
    small = type(cfg)(**{**cfg.__dict__, "grid": (4, 16, 32)})       # L = 2048, same recipe
    t = wl.head_tensors(small, 0, names=("Q", "K", "V"))
    rows = np.arange(0, small.L, 64)
    k = small.L // 16
    I = np.eye(small.d, dtype=np.float32)
    idx = oracle.lowrank_topk(t["Q"][rows], t["K"], I, I, k, "f32")     # exact top-k of q.k
    _, lse_sel = oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], idx, small.scale)
    _, lse_all = oracle.sparse_fwd(t["Q"][rows], t["K"], t["V"], np.tile(np.arange(small.L, dtype=np.int32), (len(rows), 1)), small.scale)
    mass = np.exp(lse_sel - lse_all)
    assert 0.80 < mass.mean() < 0.97, mass.mean()
