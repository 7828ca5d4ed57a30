"""Host-side checks of the synthetic workload generators and of the sizes the paper prints."""
import os

import numpy as np

import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_sizes.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            name, val, tol = line.split()
            out[name] = (float(val), float(tol))
    return out


def test_paper_size_figures():
    g = _golden()
    val, tol = g["score_tensor_bytes_H16_S100k_bf16"]
    assert abs(16 * 100_000 ** 2 * 2 - val) <= tol * val
    val, tol = g["kv_index_bytes_S50k_sparsity80"]
    L, k = 50_000, 10_000                                   # 80 % sparsity: 20 % of the keys kept
    off = wl.idx_offsets(1, 1, L, [k])
    assert abs(int(off[-1]) * np.dtype(np.int32).itemsize - val) <= tol * val


def test_configs_match_the_benchmark_list():
    Ls = [c.L for c in wl.CONFIGS]
    assert Ls == [1024, 32768, 131072, 65536, 524288]
    assert [c.H for c in wl.CONFIGS] == [2, 24, 6, 24, 2]
    assert [c.k for c in wl.CONFIGS] == [128, 2048, 8192, None, 16384]
    assert [c.r for c in wl.CONFIGS] == [16, 16, 16, 32, 32]
    ks = wl.k_per_head(wl.get_config(3))
    assert ks.shape == (24,) and set(ks.tolist()) <= {512, 1024, 2048, 4096, 8192, 16384}
    assert np.array_equal(ks, wl.k_per_head(wl.get_config(3)))       # seeded


def test_generator_is_seeded_and_rounded():
    cfg = wl.get_config(0)
    a = wl.head_tensors(cfg, 1)
    b = wl.head_tensors(cfg, 1)
    assert all(np.array_equal(a[n], b[n]) for n in a)
    assert not np.array_equal(a["Q"], wl.head_tensors(cfg, 0)["Q"])
    cfg1 = type(cfg)(**{**wl.get_config(1).__dict__, "grid": (2, 8, 16)})
    t = wl.head_tensors(cfg1, 0, names=("Q", "V"))
    assert not np.any(t["Q"].view(np.uint32) & 0xFFFF) and not np.any(t["V"].view(np.uint32) & 0xFFFF)
    assert 0.9 < t["Q"].std() < 1.1


def test_progression_index_sets_are_valid_and_invertible():
    L, k = 512, 40
    p = wl.progression_params(L, seed=3, head=2)
    rows = wl.progression_idx_rows(L, k, np.arange(L), p)
    assert rows.min() >= 0 and rows.max() < L and np.all(np.diff(rows, axis=1) > 0)
    for key in (0, 100, 511):
        assert np.array_equal(wl.progression_queries_of_key(L, k, key, p), np.nonzero((rows == key).any(axis=1))[0])


def test_random_subsets_are_distinct():
    idx = wl.random_subset_idx(100, 17, 50, seed=1)
    assert all(len(set(r.tolist())) == 17 for r in idx) and idx.min() >= 0 and idx.max() < 100
