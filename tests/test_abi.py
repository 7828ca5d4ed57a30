"""CPU-side checks of the boundary: the library loads, exports every symbol the header declares,
and turns bad arguments into error codes on the host before anything touches a GPU."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def dsv():
    import paper_2502_07590_amd as m
    if not os.path.exists(m.library_path()):
        from paper_2502_07590_amd.build import build_library
        build_library()
    m.load_library()
    return m


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dsv.h")).read()
    return sorted(set(re.findall(r"DSV_API[^;(]*?\b(dsv_\w+)\s*\(", text)))


def test_header_symbols_are_exported(dsv):
    declared = _declared_symbols()
    assert len(declared) >= 11
    lib = ctypes.CDLL(dsv.library_path())
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in include/dsv.h but not exported"
    assert sorted(dsv.EXPORTED_SYMBOLS) == declared


def test_version_and_status_strings(dsv):
    assert "gfx950" in dsv.version()
    lib = dsv.load_library()
    assert lib.dsv_status_string(0) == b"ok"
    assert all(lib.dsv_status_string(s) not in (b"ok", b"unknown status") for s in (-1, -2, -3, -4))


def test_idx_offsets_ragged(dsv):
    p = dsv.Problem(2, 3, 100, 64, 16, "bf16", [10, 100, 1], 0.1)
    assert dsv.idx_offsets(p) == [0, 1000, 11000, 11100, 12100, 22100, 22200]
    assert p.nnz == 22200


def test_bad_descriptors_are_rejected_on_the_host(dsv):
    lib = dsv.load_library()
    one = ctypes.c_void_p(256)       # a non-null, aligned placeholder: never dereferenced on these paths
    def topk(p, ws=one, ws_bytes=1 << 40):
        return lib.dsv_lowrank_topk(p.c, one, one, one, one, one, ws, ws_bytes, None)
    ok = dict(B=1, H=2, L=64, d=64, r=16, dtype="bf16", k_per_head=[8, 8], scale=0.1)
    assert topk(dsv.Problem(**{**ok, "k_per_head": [8, 65]})) == -1        # k > L
    assert topk(dsv.Problem(**{**ok, "k_per_head": [0, 8]})) == -1         # k < 1
    assert topk(dsv.Problem(**{**ok, "L": 0})) == -1
    assert topk(dsv.Problem(**{**ok, "d": 80})) == -2
    assert topk(dsv.Problem(**{**ok, "r": 12})) == -2
    assert topk(dsv.Problem(**{**ok, "dtype": __import__("torch").float16})) == -2
    assert topk(dsv.Problem(**{**ok, "L": 1 << 25, "d": 128, "k_per_head": [8, 8]})) == -2   # a head's matrix >= 4 GB
    assert topk(dsv.Problem(**{**ok, "L": (1 << 25) - 1, "d": 64, "k_per_head": [8, 8]}), ws_bytes=0) == -3   # just below: accepted
    p = dsv.Problem(**ok)
    need = dsv.lowrank_topk_workspace(p)
    assert need > 0
    assert topk(p, ws=one, ws_bytes=need - 1) == -3                         # too small
    assert topk(p, ws=None) == -3                                           # missing
    assert topk(p, ws=ctypes.c_void_p(264)) == -3                           # misaligned
    assert lib.dsv_lowrank_topk(p.c, None, one, one, one, one, one, 1 << 40, None) == -1
    assert lib.dsv_lowrank_topk(p.c, ctypes.c_void_p(260), one, one, one, one, one, 1 << 40, None) == -1
    assert lib.dsv_sparse_attn_fwd(p.c, one, one, None, one, one, one, None, 0, None) == -1
    assert lib.dsv_sparse_attn_bwd(p.c, one, one, one, one, one, one, one, one, one, one, None, 0, None) == -3
    assert dsv.sparse_attn_bwd_workspace(p) >= p.nnz * 4      # holds the transposed index
    assert lib.dsv_lowrank_scores_rows(p.c, one, one, 0, 2, one, 4, one, None) == -1   # head out of range
    # more (batch, head) pairs than a launch grid can index: an argument error, found on the host
    assert topk(dsv.Problem(**{**ok, "B": 32768, "H": 2})) == -1
    assert topk(dsv.Problem(**{**ok, "B": 1, "H": 65536, "k_per_head": [8] * 65536})) == -1
    # debug validator: descriptor, pointer and workspace errors come back before anything is launched
    lib.dsv_idx_validate_workspace.restype = ctypes.c_size_t
    assert lib.dsv_idx_validate_workspace(p.c) == 256
    assert lib.dsv_idx_validate(p.c, None, None, one, 256, None) == -1
    assert lib.dsv_idx_validate(p.c, one, None, None, 0, None) == -3
    assert lib.dsv_idx_validate(p.c, one, None, one, 255, None) == -3
    big = dsv.Problem(**{**ok, "L": 1 << 20, "k_per_head": [8, 8]})                 # unsorted rows: bitmap of L bits
    assert lib.dsv_idx_validate(big.c, one, None, one, 256, None) == -2


def test_missing_library_is_loud(dsv, monkeypatch):
    import paper_2502_07590_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", os.path.join(ROOT, "no_such_dir", "libdsv.so"))
    with pytest.raises(b.DsvError):
        b.load_library()


def test_workspace_sizes_follow_the_documented_layout(dsv):
    """Without the sorted-index flag stage 2 needs no scratch; with it, segment pointers, the row order per
    range and the fp32 partial results -- sizes that can be re-derived from the plan the header describes
    (ranges of about 2 MB of K+V rows for the forward, 4 MB for the backward steps, a multiple of 8)."""
    import workloads as wl
    cfg = wl.get_config(2)
    ks = [int(k) for k in wl.k_per_head(cfg)]
    plain = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, ks, cfg.scale)
    flagged = dsv.Problem(1, cfg.H, cfg.L, cfg.d, cfg.r, cfg.dtype, ks, cfg.scale, sorted_index=True)
    assert dsv.sparse_attn_fwd_workspace(plain) == 0
    assert dsv.sparse_attn_bwd_dq_workspace(plain) == 0
    assert dsv.sparse_attn_bwd_dkdv_workspace(plain) == 0
    rows = cfg.H * cfg.L

    def ranges(target_bytes):
        target_rows = target_bytes // (2 * cfg.d * 2)
        return -(-cfg.L // (8 * target_rows)) * 8

    s_fwd, s_bwd = ranges(2 << 20), ranges(4 << 20)
    assert (s_fwd, s_bwd) == (32, 16)
    fwd = dsv.sparse_attn_fwd_workspace(flagged)
    partial = rows * s_fwd * cfg.d * 4
    assert partial < fwd < partial + rows * (s_fwd + 1) * 4 * 5 + (1 << 20)       # + seg, m, l, order, counters
    step = dsv.sparse_attn_bwd_dq_workspace(flagged)
    assert step == dsv.sparse_attn_bwd_dkdv_workspace(flagged)            # the two steps share one layout
    partial = 2 * rows * s_bwd * cfg.d * 4
    assert partial < step < partial + rows * (s_bwd + 1) * 4 * 5 + rows * 8 + (1 << 20)   # + seg, Delta parts, order, ...
    # whole backward with its own transpose also holds Delta, the transposed index and its column pointers
    assert dsv.sparse_attn_bwd_workspace(flagged) >= step + flagged.nnz * 4 + cfg.H * (cfg.L + 1) * 8 + rows * 4
    assert dsv.sparse_attn_bwd_t_workspace(flagged) >= step + rows * 4
    # stage 1: low-rank projections plus a few words of selection state per query and key
    s1 = dsv.lowrank_topk_t_workspace(flagged)
    assert 2 * rows * cfg.r * 2 < s1 < 2 * rows * cfg.r * 2 + rows * 4 * 8


def test_measurement_aid_rejects_what_has_not_run(dsv):
    lib = dsv.load_library()
    ms = ctypes.c_float(-1.0)
    assert lib.dsv_kernel_timing(0) == 0                                   # switching it off touches no GPU
    for span in range(len(dsv.KERNEL_SPANS)):
        assert lib.dsv_kernel_ms(span, ctypes.byref(ms)) == -1            # nothing recorded
    assert lib.dsv_kernel_ms(-1, ctypes.byref(ms)) == -1
    assert lib.dsv_kernel_ms(len(dsv.KERNEL_SPANS), ctypes.byref(ms)) == -1
    assert lib.dsv_kernel_ms(0, None) == -1
    assert ms.value == -1.0


def test_threshold_search_choice_is_host_arithmetic(dsv):
    """dsv_threshold_search / dsv_threshold_sample_keys: which heads the windowed threshold search takes, and with how
    large a key sample (no GPU involved)."""
    try:
        assert dsv.threshold_search(0) in (0, 1, 2)
        n = dsv.threshold_sample_keys(131072, 8192)
        assert n == 2080                                   # (L sqrt(f (1 - f)) / 700)^2 = 2054.4, up to a multiple of 32
        assert dsv.threshold_sample_keys(524288, 16384) == 16384             # capped: min(L / 8, 16384)
        assert dsv.threshold_sample_keys(65536, 512) == 8192                 # 64 sample keys above the threshold: 64 L / k
        assert dsv.threshold_sample_keys(8192, 512) == 0                     # short sequence
        assert dsv.threshold_sample_keys(131072, 32769) == 0                 # k > L / 4: threshold too close to zero
        assert dsv.threshold_sample_keys(131072, 64) == 0                    # no sample of <= L / 8 keys holds the upper bound
        assert dsv.threshold_sample_keys(131072, 131072) == 0 and dsv.threshold_sample_keys(131072, 0) == 0
        for L, k in ((131072, 8192), (65536, 1024), (32768, 8192), (1 << 20, 4096)):
            n = dsv.threshold_sample_keys(L, k)
            assert n % 32 == 0 and 2048 <= n <= min(L // 8, 16384)
        assert dsv.threshold_search(2) == 0
        assert dsv.threshold_sample_keys(4096, 256) == 2048                  # forced: up to L / 2 keys
        assert dsv.threshold_sample_keys(4000, 256) == 0                     # below twice the smallest sample
        assert dsv.threshold_sample_keys(8192, 4096) == 2048                 # forced: any density the sample can bracket
        assert dsv.threshold_sample_keys(8192, 1) == 0
        assert dsv.threshold_search(1) == 2
        assert dsv.threshold_sample_keys(131072, 8192) == 0
        with pytest.raises(ValueError):
            dsv.threshold_search(3)
        assert dsv.load_library().dsv_threshold_search(-1) == -1
        assert dsv.threshold_search(1) == 1                                  # the refused calls changed nothing
    finally:
        dsv.threshold_search(0)
