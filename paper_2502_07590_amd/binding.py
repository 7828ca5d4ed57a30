"""ctypes binding of libdsv.so: same names as the C entry points, argument marshalling only.

PyTorch supplies device memory (tensor.data_ptr()) and the HIP stream; nothing here computes.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# DSV_LIBRARY: load another build of the same library (tuning builds); default: the in-tree build
_LIB_PATH = os.environ.get("DSV_LIBRARY") or os.path.join(_PKG, "libdsv.so")

DSV_F32, DSV_BF16 = 0, 1
DSV_FLAG_SORTED_INDEX = 1
_DTYPE_CODE = {torch.float32: DSV_F32, torch.bfloat16: DSV_BF16}
_DTYPE_NAME = {"f32": torch.float32, "bf16": torch.bfloat16}

EXPORTED_SYMBOLS = (
    "dsv_version", "dsv_status_string", "dsv_idx_offsets",
    "dsv_lowrank_topk_workspace", "dsv_lowrank_topk", "dsv_lowrank_topk_t_workspace", "dsv_lowrank_topk_t",
    "dsv_sparse_attn_fwd_workspace", "dsv_sparse_attn_fwd",
    "dsv_sparse_attn_bwd_workspace", "dsv_sparse_attn_bwd",
    "dsv_sparse_attn_bwd_t_workspace", "dsv_sparse_attn_bwd_t",
    "dsv_sparse_attn_bwd_dq_workspace", "dsv_sparse_attn_bwd_dq", "dsv_idx_transpose_workspace", "dsv_idx_transpose",
    "dsv_sparse_attn_bwd_dkdv_workspace", "dsv_sparse_attn_bwd_dkdv",
    "dsv_idx_validate_workspace", "dsv_idx_validate",
    "dsv_predictor_loss_workspace", "dsv_predictor_loss", "dsv_profile_sparsity_workspace", "dsv_profile_sparsity",
    "dsv_lowrank_topk_grouped_workspace", "dsv_lowrank_topk_grouped", "dsv_sparse_attn_fwd_grouped_workspace",
    "dsv_sparse_attn_fwd_grouped",
    "dsv_sparse_attn_bwd_grouped_workspace", "dsv_sparse_attn_bwd_grouped",
    "dsv_group_overlap_workspace", "dsv_group_overlap", "dsv_choose_grouping_workspace", "dsv_choose_grouping",
    "dsv_lowrank_topk_noalloc_max_bytes", "dsv_lowrank_topk_noalloc",
    "dsv_lowrank_project", "dsv_lowrank_scores_rows",
    "dsv_kernel_timing", "dsv_kernel_ms", "dsv_threshold_search", "dsv_threshold_sample_keys", "dsv_measure_gather_ceiling",
)


class DsvError(RuntimeError):
    pass


class _CProblem(ctypes.Structure):
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("L", ctypes.c_int32), ("d", ctypes.c_int32),
                ("r", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("k_per_head", ctypes.POINTER(ctypes.c_int32)), ("scale", ctypes.c_float),
                ("flags", ctypes.c_uint32)]


class _CGrouping(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("F", "Hh", "Ww", "gf", "gh", "gw")]


class Grouping:
    """Token grid (frames, height, width) and the cube that forms a query group (mirrors struct dsv_grouping)."""

    def __init__(self, grid, cube):
        self.grid, self.cube = tuple(int(x) for x in grid), tuple(int(x) for x in cube)
        self._c = _CGrouping(*self.grid, *self.cube)

    @property
    def c(self):
        return ctypes.byref(self._c)

    @property
    def G(self) -> int:
        return self.cube[0] * self.cube[1] * self.cube[2]


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libdsv.so from the package directory.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise DsvError(f"{_LIB_PATH} is missing: build it with `python -m paper_2502_07590_amd.build` "
                       "(there is no fallback path)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz, i32 = ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int32
    P = ctypes.POINTER(_CProblem)
    lib.dsv_version.restype = ctypes.c_char_p
    lib.dsv_status_string.restype = ctypes.c_char_p
    lib.dsv_status_string.argtypes = [ctypes.c_int]
    lib.dsv_idx_offsets.restype = ctypes.c_int
    lib.dsv_idx_offsets.argtypes = [P, ctypes.POINTER(ctypes.c_int64)]
    for name in ("dsv_lowrank_topk_workspace", "dsv_sparse_attn_fwd_workspace", "dsv_sparse_attn_bwd_workspace",
                 "dsv_idx_transpose_workspace", "dsv_lowrank_topk_t_workspace", "dsv_sparse_attn_bwd_t_workspace",
                 "dsv_sparse_attn_bwd_dq_workspace", "dsv_sparse_attn_bwd_dkdv_workspace",
                 "dsv_idx_validate_workspace", "dsv_group_overlap_workspace", "dsv_choose_grouping_workspace"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [P]
    lib.dsv_lowrank_topk.restype = ctypes.c_int
    lib.dsv_lowrank_topk.argtypes = [P, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_lowrank_topk_t.restype = ctypes.c_int
    lib.dsv_lowrank_topk_t.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_fwd.restype = ctypes.c_int
    lib.dsv_sparse_attn_fwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_bwd.restype = ctypes.c_int
    lib.dsv_sparse_attn_bwd.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_bwd_dq.restype = ctypes.c_int
    lib.dsv_sparse_attn_bwd_dq.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_bwd_t.restype = ctypes.c_int
    lib.dsv_sparse_attn_bwd_t.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_idx_transpose.restype = ctypes.c_int
    lib.dsv_idx_transpose.argtypes = [P, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_bwd_dkdv.restype = ctypes.c_int
    lib.dsv_sparse_attn_bwd_dkdv.argtypes = [P, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_lowrank_topk_noalloc_max_bytes.restype = sz
    lib.dsv_lowrank_topk_noalloc_max_bytes.argtypes = []
    lib.dsv_lowrank_topk_noalloc.restype = ctypes.c_int
    lib.dsv_lowrank_topk_noalloc.argtypes = [P, vp, vp, vp, vp, vp, vp]
    PG = ctypes.POINTER(_CGrouping)
    for name in ("dsv_lowrank_topk_grouped_workspace", "dsv_sparse_attn_bwd_grouped_workspace",
                 "dsv_sparse_attn_fwd_grouped_workspace"):
        getattr(lib, name).restype = sz
        getattr(lib, name).argtypes = [P, PG]
    lib.dsv_lowrank_topk_grouped.restype = ctypes.c_int
    lib.dsv_lowrank_topk_grouped.argtypes = [P, PG, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_fwd_grouped.restype = ctypes.c_int
    lib.dsv_sparse_attn_fwd_grouped.argtypes = [P, PG, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.dsv_sparse_attn_bwd_grouped.restype = ctypes.c_int
    lib.dsv_sparse_attn_bwd_grouped.argtypes = [P, PG] + [vp] * 12 + [vp, sz, vp]
    lib.dsv_group_overlap.restype = ctypes.c_int
    lib.dsv_group_overlap.argtypes = [P, PG, vp, vp, vp, sz, vp]
    lib.dsv_choose_grouping.restype = ctypes.c_int
    lib.dsv_choose_grouping.argtypes = [P, i32, i32, i32, ctypes.POINTER(ctypes.c_int32), i32, vp, ctypes.c_float,
                                        ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float), vp, sz, vp]
    lib.dsv_profile_sparsity_workspace.restype = sz
    lib.dsv_profile_sparsity_workspace.argtypes = [P, i32]
    lib.dsv_profile_sparsity.restype = ctypes.c_int
    lib.dsv_profile_sparsity.argtypes = [P, vp, vp, vp, i32, ctypes.c_float, vp, vp, vp, ctypes.c_float, vp, sz, vp]
    lib.dsv_predictor_loss_workspace.restype = sz
    lib.dsv_predictor_loss_workspace.argtypes = [P, i32]
    lib.dsv_predictor_loss.restype = ctypes.c_int
    lib.dsv_predictor_loss.argtypes = [P, vp, vp, vp, vp, vp, i32, vp, vp, vp, vp, sz, vp]
    lib.dsv_idx_validate.restype = ctypes.c_int
    lib.dsv_idx_validate.argtypes = [P, vp, ctypes.POINTER(ctypes.c_int64), vp, sz, vp]
    lib.dsv_lowrank_project.restype = ctypes.c_int
    lib.dsv_lowrank_project.argtypes = [P, vp, vp, vp, vp, vp, vp, vp]
    lib.dsv_lowrank_scores_rows.restype = ctypes.c_int
    lib.dsv_lowrank_scores_rows.argtypes = [P, vp, vp, i32, i32, vp, i32, vp, vp]
    lib.dsv_threshold_sample_keys.restype = ctypes.c_int32
    lib.dsv_threshold_sample_keys.argtypes = [i32, i32]
    lib.dsv_threshold_search.restype = ctypes.c_int32
    lib.dsv_threshold_search.argtypes = [i32]
    lib.dsv_kernel_timing.restype = ctypes.c_int
    lib.dsv_kernel_timing.argtypes = [i32]
    lib.dsv_kernel_ms.restype = ctypes.c_int
    lib.dsv_kernel_ms.argtypes = [i32, ctypes.POINTER(ctypes.c_float)]
    lib.dsv_measure_gather_ceiling.restype = ctypes.c_int
    lib.dsv_measure_gather_ceiling.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, i32, ctypes.POINTER(ctypes.c_float), vp]
    _lib = lib
    return lib


def version() -> str:
    return load_library().dsv_version().decode()


def _check(status: int, what: str):
    if status != 0:
        msg = load_library().dsv_status_string(status).decode()
        raise DsvError(f"{what} failed: {msg} (status {status})")


class Problem:
    """Host-side problem descriptor (mirrors struct dsv_problem)."""

    def __init__(self, B: int, H: int, L: int, d: int, r: int, dtype, k_per_head: Sequence[int], scale: float,
                 sorted_index: bool = False):
        if isinstance(dtype, str):
            dtype = _DTYPE_NAME[dtype]
        self.B, self.H, self.L, self.d, self.r = int(B), int(H), int(L), int(d), int(r)
        self.torch_dtype = dtype
        self.k_per_head = [int(k) for k in k_per_head]
        self.scale = float(scale)
        self._k_arr = (ctypes.c_int32 * len(self.k_per_head))(*self.k_per_head)
        self._c = _CProblem(self.B, self.H, self.L, self.d, self.r, _DTYPE_CODE.get(dtype, -1),
                            ctypes.cast(self._k_arr, ctypes.POINTER(ctypes.c_int32)), self.scale,
                            DSV_FLAG_SORTED_INDEX if sorted_index else 0)
        self.sorted_index = bool(sorted_index)

    @property
    def c(self):
        return ctypes.byref(self._c)

    @property
    def nnz(self) -> int:
        return self.B * self.L * sum(self.k_per_head)


def idx_offsets(p: Problem):
    off = (ctypes.c_int64 * (p.B * p.H + 1))()
    _check(load_library().dsv_idx_offsets(p.c, off), "dsv_idx_offsets")
    return list(off)


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda:
        raise DsvError("libdsv takes device tensors")
    if not t.is_contiguous():
        raise DsvError("libdsv takes contiguous tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(nbytes: int, device, workspace, stream=None):
    if nbytes == 0 and workspace is None:
        return None, 0
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
        if stream is not None:
            # scratch made here dies when the wrapper returns, while the kernels may still be pending on the
            # caller's stream: tell the caching allocator, so that it does not hand the block out under them
            workspace.record_stream(stream)
    return workspace, workspace.numel() * workspace.element_size()


def lowrank_topk_workspace(p: Problem) -> int:
    return int(load_library().dsv_lowrank_topk_workspace(p.c))


def sparse_attn_fwd_workspace(p: Problem) -> int:
    return int(load_library().dsv_sparse_attn_fwd_workspace(p.c))


def sparse_attn_bwd_workspace(p: Problem) -> int:
    return int(load_library().dsv_sparse_attn_bwd_workspace(p.c))


def lowrank_topk(p: Problem, Q, K, Wq, Wk, idx=None, workspace=None, stream=None):
    """idx (int32, ragged [sum_h L*k_h]) = per-(head, query) top-k keys of the low-rank scores."""
    lib = load_library()
    if idx is None:
        idx = torch.empty(p.nnz, dtype=torch.int32, device=Q.device)
    ws, nbytes = _workspace(lowrank_topk_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_lowrank_topk(p.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(idx), _ptr(ws), nbytes,
                                _stream(stream)), "dsv_lowrank_topk")
    return idx


def lowrank_topk_noalloc_max_bytes() -> int:
    return int(load_library().dsv_lowrank_topk_noalloc_max_bytes())


def lowrank_topk_noalloc(p: Problem, Q, K, Wq, Wk, idx, stream=None):
    """dsv_lowrank_topk with the scratch inside the library: the caller passes inputs and the output only."""
    _check(load_library().dsv_lowrank_topk_noalloc(p.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(idx),
                                                   _stream(stream)), "dsv_lowrank_topk_noalloc")
    return idx


def lowrank_topk_t_workspace(p: Problem) -> int:
    return int(load_library().dsv_lowrank_topk_t_workspace(p.c))


def lowrank_topk_t(p: Problem, Q, K, Wq, Wk, idx=None, idx_t=None, col_ptr=None, workspace=None, stream=None):
    """Stage 1 plus the transposed index: (idx, idx_t, col_ptr)."""
    lib = load_library()
    idx = torch.empty(p.nnz, dtype=torch.int32, device=Q.device) if idx is None else idx
    idx_t = torch.empty(p.nnz, dtype=torch.int32, device=Q.device) if idx_t is None else idx_t
    col_ptr = torch.empty((p.B * p.H, p.L + 1), dtype=torch.int64, device=Q.device) if col_ptr is None else col_ptr
    ws, nbytes = _workspace(lowrank_topk_t_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_lowrank_topk_t(p.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(idx), _ptr(idx_t), _ptr(col_ptr),
                                  _ptr(ws), nbytes, _stream(stream)), "dsv_lowrank_topk_t")
    return idx, idx_t, col_ptr


def sparse_attn_fwd(p: Problem, Q, K, V, idx, O=None, lse=None, workspace=None, stream=None):
    lib = load_library()
    if O is None:
        O = torch.empty_like(Q)
    if lse is None:
        lse = torch.empty((p.B, p.H, p.L), dtype=torch.float32, device=Q.device)
    ws, nbytes = _workspace(sparse_attn_fwd_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_sparse_attn_fwd(p.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O), _ptr(lse), _ptr(ws), nbytes,
                                   _stream(stream)), "dsv_sparse_attn_fwd")
    return O, lse


def sparse_attn_bwd(p: Problem, Q, K, V, idx, O, lse, dO, dQ=None, dK=None, dV=None, workspace=None, stream=None):
    lib = load_library()
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    ws, nbytes = _workspace(sparse_attn_bwd_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_sparse_attn_bwd(p.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O), _ptr(lse), _ptr(dO),
                                   _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws), nbytes, _stream(stream)),
           "dsv_sparse_attn_bwd")
    return dQ, dK, dV


def sparse_attn_bwd_dq_workspace(p: Problem) -> int:
    return int(load_library().dsv_sparse_attn_bwd_dq_workspace(p.c))


def sparse_attn_bwd_dq(p: Problem, Q, K, V, idx, O, lse, dO, dQ=None, delta=None, workspace=None, stream=None):
    lib = load_library()
    dQ = torch.empty_like(Q) if dQ is None else dQ
    delta = torch.empty((p.B, p.H, p.L), dtype=torch.float32, device=Q.device) if delta is None else delta
    ws, nbytes = _workspace(sparse_attn_bwd_dq_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_sparse_attn_bwd_dq(p.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(O), _ptr(lse), _ptr(dO),
                                      _ptr(dQ), _ptr(delta), _ptr(ws), nbytes, _stream(stream)),
           "dsv_sparse_attn_bwd_dq")
    return dQ, delta


def sparse_attn_bwd_t_workspace(p: Problem) -> int:
    return int(load_library().dsv_sparse_attn_bwd_t_workspace(p.c))


def sparse_attn_bwd_t(p: Problem, Q, K, V, idx, idx_t, col_ptr, O, lse, dO, dQ=None, dK=None, dV=None,
                      workspace=None, stream=None):
    lib = load_library()
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    ws, nbytes = _workspace(sparse_attn_bwd_t_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_sparse_attn_bwd_t(p.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx), _ptr(idx_t), _ptr(col_ptr), _ptr(O),
                                     _ptr(lse), _ptr(dO), _ptr(dQ), _ptr(dK), _ptr(dV), _ptr(ws), nbytes,
                                     _stream(stream)), "dsv_sparse_attn_bwd_t")
    return dQ, dK, dV


def idx_transpose_workspace(p: Problem) -> int:
    return int(load_library().dsv_idx_transpose_workspace(p.c))


def idx_transpose(p: Problem, idx, idx_t=None, col_ptr=None, workspace=None, stream=None):
    lib = load_library()
    idx_t = torch.empty_like(idx) if idx_t is None else idx_t
    col_ptr = torch.empty((p.B * p.H, p.L + 1), dtype=torch.int64, device=idx.device) if col_ptr is None else col_ptr
    ws, nbytes = _workspace(idx_transpose_workspace(p), idx.device, workspace, stream)
    _check(lib.dsv_idx_transpose(p.c, _ptr(idx), _ptr(idx_t), _ptr(col_ptr), _ptr(ws), nbytes, _stream(stream)),
           "dsv_idx_transpose")
    return idx_t, col_ptr


def sparse_attn_bwd_dkdv_workspace(p: Problem) -> int:
    return int(load_library().dsv_sparse_attn_bwd_dkdv_workspace(p.c))


def sparse_attn_bwd_dkdv(p: Problem, Q, K, V, idx_t, col_ptr, lse, delta, dO, dK=None, dV=None, workspace=None,
                         stream=None):
    lib = load_library()
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    ws, nbytes = _workspace(sparse_attn_bwd_dkdv_workspace(p), Q.device, workspace, stream)
    _check(lib.dsv_sparse_attn_bwd_dkdv(p.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx_t), _ptr(col_ptr), _ptr(lse),
                                        _ptr(delta), _ptr(dO), _ptr(dK), _ptr(dV), _ptr(ws), nbytes, _stream(stream)),
           "dsv_sparse_attn_bwd_dkdv")
    return dK, dV


# ---- query grouping -------------------------------------------------------------------------------
def lowrank_topk_grouped_workspace(p: Problem, g: Grouping) -> int:
    return int(load_library().dsv_lowrank_topk_grouped_workspace(p.c, g.c))


def lowrank_topk_grouped(p: Problem, g: Grouping, Q, K, Wq, Wk, transposed=True, idx_g=None, idx_t_g=None, col_ptr=None,
                         workspace=None, stream=None):
    """Stage 1 on the groups' centre queries: (idx_g, idx_t_g, col_ptr); the last two None if not transposed."""
    lib = load_library()
    n = p.nnz // g.G
    idx_g = torch.empty(n, dtype=torch.int32, device=Q.device) if idx_g is None else idx_g
    if transposed:
        idx_t_g = torch.empty(n, dtype=torch.int32, device=Q.device) if idx_t_g is None else idx_t_g
        col_ptr = torch.empty((p.B * p.H, p.L + 1), dtype=torch.int64, device=Q.device) if col_ptr is None else col_ptr
    ws, nbytes = _workspace(lowrank_topk_grouped_workspace(p, g), Q.device, workspace, stream)
    _check(lib.dsv_lowrank_topk_grouped(p.c, g.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(idx_g),
                                        _ptr(idx_t_g) if transposed else None, _ptr(col_ptr) if transposed else None,
                                        _ptr(ws), nbytes, _stream(stream)), "dsv_lowrank_topk_grouped")
    return idx_g, (idx_t_g if transposed else None), (col_ptr if transposed else None)


def sparse_attn_fwd_grouped_workspace(p: Problem, g: Grouping) -> int:
    return int(load_library().dsv_sparse_attn_fwd_grouped_workspace(p.c, g.c))


def sparse_attn_fwd_grouped(p: Problem, g: Grouping, Q, K, V, idx_g, O=None, lse=None, workspace=None, stream=None):
    O = torch.empty_like(Q) if O is None else O
    lse = torch.empty((p.B, p.H, p.L), dtype=torch.float32, device=Q.device) if lse is None else lse
    ws, nbytes = _workspace(sparse_attn_fwd_grouped_workspace(p, g), Q.device, workspace, stream)
    _check(load_library().dsv_sparse_attn_fwd_grouped(p.c, g.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx_g), _ptr(O), _ptr(lse),
                                                      _ptr(ws), nbytes, _stream(stream)), "dsv_sparse_attn_fwd_grouped")
    return O, lse


def sparse_attn_bwd_grouped_workspace(p: Problem, g: Grouping) -> int:
    return int(load_library().dsv_sparse_attn_bwd_grouped_workspace(p.c, g.c))


def sparse_attn_bwd_grouped(p: Problem, g: Grouping, Q, K, V, idx_g, idx_t_g, col_ptr, O, lse, dO, dQ=None, dK=None,
                            dV=None, workspace=None, stream=None):
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(V) if dV is None else dV
    ws, nbytes = _workspace(sparse_attn_bwd_grouped_workspace(p, g), Q.device, workspace, stream)
    _check(load_library().dsv_sparse_attn_bwd_grouped(p.c, g.c, _ptr(Q), _ptr(K), _ptr(V), _ptr(idx_g), _ptr(idx_t_g),
                                                      _ptr(col_ptr), _ptr(O), _ptr(lse), _ptr(dO), _ptr(dQ), _ptr(dK),
                                                      _ptr(dV), _ptr(ws), nbytes, _stream(stream)),
           "dsv_sparse_attn_bwd_grouped")
    return dQ, dK, dV


# ---- predictor side -------------------------------------------------------------------------------
def group_overlap(p: Problem, g: Grouping, idx, overlap=None, workspace=None, stream=None):
    """Share of the queries' own selections (per-query idx) that their group centre's row holds: float [B*H]."""
    lib = load_library()
    overlap = torch.empty(p.B * p.H, dtype=torch.float32, device=idx.device) if overlap is None else overlap
    ws, nbytes = _workspace(int(lib.dsv_group_overlap_workspace(p.c)), idx.device, workspace, stream)
    _check(lib.dsv_group_overlap(p.c, g.c, _ptr(idx), _ptr(overlap), _ptr(ws), nbytes, _stream(stream)), "dsv_group_overlap")
    return overlap


def choose_grouping(p: Problem, grid, cubes, idx, min_overlap: float = 0.8, workspace=None, stream=None):
    """Largest candidate cube whose overlap reaches min_overlap in every head: (index into cubes or -1, overlaps
    [len(cubes), B*H] as nested lists; -1 rows for cubes that do not tile the grid).  Waits for the stream."""
    lib = load_library()
    n = len(cubes)
    flat = (ctypes.c_int32 * (3 * n))(*[int(x) for c in cubes for x in c])
    chosen = ctypes.c_int32(-2)
    out = (ctypes.c_float * (n * p.B * p.H))()
    ws, nbytes = _workspace(int(lib.dsv_choose_grouping_workspace(p.c)), idx.device, workspace, stream)
    _check(lib.dsv_choose_grouping(p.c, int(grid[0]), int(grid[1]), int(grid[2]), flat, n, _ptr(idx), float(min_overlap),
                                   ctypes.byref(chosen), out, _ptr(ws), nbytes, _stream(stream)), "dsv_choose_grouping")
    nbh = p.B * p.H
    return int(chosen.value), [[float(out[c * nbh + e]) for e in range(nbh)] for c in range(n)]


def predictor_loss_workspace(p: Problem, n_rows: int) -> int:
    return int(load_library().dsv_predictor_loss_workspace(p.c, int(n_rows)))


def predictor_loss(p: Problem, Q, K, Wq, Wk, rows, workspace=None, stream=None):
    """(loss [B*H, 3] = {total, cos, norm}, dWq [B*H, d, r], dWk [B*H, d, r]) on the sampled query rows."""
    n = int(rows.numel())
    dev = Q.device
    loss = torch.empty((p.B * p.H, 3), dtype=torch.float32, device=dev)
    dWq = torch.empty((p.B * p.H, p.d, p.r), dtype=torch.float32, device=dev)
    dWk = torch.empty((p.B * p.H, p.d, p.r), dtype=torch.float32, device=dev)
    ws, nbytes = _workspace(predictor_loss_workspace(p, n), dev, workspace, stream)
    _check(load_library().dsv_predictor_loss(p.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(rows), n, _ptr(loss), _ptr(dWq),
                                             _ptr(dWk), _ptr(ws), nbytes, _stream(stream)), "dsv_predictor_loss")
    return loss, dWq, dWk


def profile_sparsity(p: Problem, Q, K, rows, mass: float = 0.9, ema=None, alpha: float = 0.1, workspace=None, stream=None):
    """(sparsity [B*H], counts [B*H, n_rows]) of the sampled query rows; `ema` ([B*H] float, optional) is updated in place."""
    n = int(rows.numel())
    dev = Q.device
    counts = torch.empty((p.B * p.H, n), dtype=torch.int32, device=dev)
    sparsity = torch.empty(p.B * p.H, dtype=torch.float32, device=dev)
    lib = load_library()
    ws, nbytes = _workspace(int(lib.dsv_profile_sparsity_workspace(p.c, n)), dev, workspace, stream)
    _check(lib.dsv_profile_sparsity(p.c, _ptr(Q), _ptr(K), _ptr(rows), n, float(mass), _ptr(counts), _ptr(sparsity), _ptr(ema),
                                    float(alpha), _ptr(ws), nbytes, _stream(stream)), "dsv_profile_sparsity")
    return sparsity, counts


def idx_validate(p: Problem, idx, workspace=None, stream=None):
    """Debug check of idx against the contract (in range, distinct, ascending if p.sorted_index).  Waits for the
    stream.  Returns (ok, (n_bad_rows, first_bad_bh, first_bad_row))."""
    lib = load_library()
    ws, nbytes = _workspace(int(lib.dsv_idx_validate_workspace(p.c)), idx.device, workspace, stream)
    rep = (ctypes.c_int64 * 3)()
    st = lib.dsv_idx_validate(p.c, _ptr(idx), rep, _ptr(ws), nbytes, _stream(stream))
    if st not in (0, -1):
        _check(st, "dsv_idx_validate")
    return st == 0, tuple(int(x) for x in rep)


def lowrank_project(p: Problem, Q, K, Wq, Wk, Qlr=None, Klr=None, stream=None):
    lib = load_library()
    shape = (p.B, p.H, p.L, p.r)
    Qlr = torch.empty(shape, dtype=p.torch_dtype, device=Q.device) if Qlr is None else Qlr
    Klr = torch.empty(shape, dtype=p.torch_dtype, device=Q.device) if Klr is None else Klr
    _check(lib.dsv_lowrank_project(p.c, _ptr(Q), _ptr(K), _ptr(Wq), _ptr(Wk), _ptr(Qlr), _ptr(Klr),
                                   _stream(stream)), "dsv_lowrank_project")
    return Qlr, Klr


def lowrank_scores_rows(p: Problem, Qlr, Klr, b: int, h: int, rows, scores=None, stream=None):
    lib = load_library()
    n = int(rows.numel())
    scores = torch.empty((n, p.L), dtype=torch.float32, device=Qlr.device) if scores is None else scores
    _check(lib.dsv_lowrank_scores_rows(p.c, _ptr(Qlr), _ptr(Klr), int(b), int(h), _ptr(rows), n, _ptr(scores),
                                       _stream(stream)), "dsv_lowrank_scores_rows")
    return scores


KERNEL_SPANS = ("fwd_sweep", "dq_sweep", "dkdv_sweep", "threshold", "emit", "emit_t_count", "emit_t_write")


def threshold_search(mode: int) -> int:
    """dsv_threshold_search: 0 automatic, 1 radix search, 2 windowed search wherever it fits; returns the old mode."""
    old = load_library().dsv_threshold_search(int(mode))
    if old < 0:
        raise ValueError(f"dsv_threshold_search: mode {mode} is not 0, 1 or 2")
    return old


def threshold_sample_keys(L: int, k: int) -> int:
    """dsv_threshold_sample_keys: keys the windowed threshold search samples for a head keeping k of L (0: radix search)."""
    return int(load_library().dsv_threshold_sample_keys(int(L), int(k)))


def kernel_timing(enable: bool):
    _check(load_library().dsv_kernel_timing(1 if enable else 0), "dsv_kernel_timing")


def kernel_ms(span: str) -> float:
    ms = ctypes.c_float(0.0)
    _check(load_library().dsv_kernel_ms(KERNEL_SPANS.index(span), ctypes.byref(ms)), "dsv_kernel_ms")
    return float(ms.value)


def measure_gather_ceiling(n_ranges: int, range_rows: int, nq: int, k: int, idx_rows: int, K, V, idx, out, reps: int = 3,
                           stream=None) -> float:
    """Mean ms per launch of the pure-gather probe (see dsv_measure_gather_ceiling)."""
    ms = ctypes.c_float(0.0)
    _check(load_library().dsv_measure_gather_ceiling(n_ranges, range_rows, nq, k, idx_rows, _ptr(K), _ptr(V), _ptr(idx),
                                                     _ptr(out), reps, ctypes.byref(ms), _stream(stream)),
           "dsv_measure_gather_ceiling")
    return float(ms.value)
