"""ctypes binding of the C-ABI library (``include/lf.h``): argument marshalling only.

Every step of the hot path runs inside the library's HIP kernels.  PyTorch is used here
for nothing but device memory (``torch.empty`` on the GPU) and the current HIP stream.
There is no CPU fallback: if the shared library has not been built, or a call returns an
error status, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "liblf_hsa.so")
_lib = None

LF_OK = 0
LF_BF16 = 0
LF_SCHED_FIXED, LF_SCHED_LINEAR, LF_SCHED_CAG = 0, 1, 2
LF_OF_CANDIDATES, LF_OF_HISTORY, LF_OF_ALL = 0, 1, 2


class lf_schedule(C.Structure):
    _fields_ = [("mode", C.c_int32), ("n_chunks", C.c_int32), ("frames_per_chunk", C.c_int32),
                ("frame_len", C.c_int32), ("block", C.c_int32), ("n_sink", C.c_int32),
                ("n_win", C.c_int32), ("k_frames", C.c_int32), ("ratio_of", C.c_int32),
                ("current_mandatory", C.c_int32), ("first_chunk_dense", C.c_int32),
                ("reserved", C.c_int32),
                ("keep_fixed", C.c_double), ("keep_first", C.c_double), ("keep_last", C.c_double),
                ("s_base", C.c_double), ("s_target", C.c_double)]


class lf_budget(C.Structure):
    _fields_ = [("n_hist_frames", C.c_int32), ("frames_per_chunk", C.c_int32),
                ("n_sink", C.c_int32), ("n_win", C.c_int32), ("k_frames", C.c_int32),
                ("k_blocks", C.c_int32), ("current_mandatory", C.c_int32), ("list_len", C.c_int32),
                ("keep_ratio", C.c_double)]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class lf_shape(C.Structure):
    _fields_ = [("heads", C.c_int32), ("head_dim", C.c_int32), ("frame_len", C.c_int32),
                ("block", C.c_int32), ("q_len", C.c_int32), ("kv_len", C.c_int32),
                ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("q_stride_tok", C.c_int64), ("q_stride_head", C.c_int64),
                ("k_stride_tok", C.c_int64), ("k_stride_head", C.c_int64),
                ("v_stride_tok", C.c_int64), ("v_stride_head", C.c_int64),
                ("o_stride_tok", C.c_int64), ("o_stride_head", C.c_int64)]


class lf_producer_shape(C.Structure):
    _fields_ = [("heads", C.c_int32), ("head_dim", C.c_int32), ("tokens", C.c_int32),
                ("across_heads", C.c_int32), ("pairing", C.c_int32), ("eps", C.c_float),
                ("x_stride_tok", C.c_int64), ("y_stride_tok", C.c_int64), ("y_stride_head", C.c_int64)]


class LfError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lf_strerror(status)} (lf_status {status})")


def library_path() -> str:
    return _LIB_PATH


def load() -> C.CDLL:
    """Load liblf_hsa.so (built by ``paper_2602_04789_amd.build``); raise if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} not found: build it with `python -m paper_2602_04789_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(_LIB_PATH)
    vp, i32p = C.c_void_p, C.POINTER(C.c_int32)
    lib.lf_chunk_budget.argtypes = [C.c_int32, C.POINTER(lf_schedule), C.POINTER(lf_budget)]
    lib.lf_chunk_budget.restype = C.c_int
    lib.lf_workspace_bytes.argtypes = [C.POINTER(lf_shape), C.POINTER(lf_budget)]
    lib.lf_workspace_bytes.restype = C.c_size_t
    lib.lf_workspace_layout.argtypes = [C.POINTER(lf_shape), C.POINTER(lf_budget),
                                        C.POINTER(C.c_size_t)]
    lib.lf_workspace_layout.restype = C.c_int
    lib.lf_select_mask.argtypes = [vp, vp, C.POINTER(lf_shape), C.POINTER(lf_budget), vp, vp,
                                   C.c_size_t, vp]
    lib.lf_select_mask.restype = C.c_int
    lib.lf_sparse_attn.argtypes = [vp, vp, vp, C.POINTER(lf_shape), vp, C.c_int32, C.c_float,
                                   vp, vp]
    lib.lf_sparse_attn.restype = C.c_int
    lib.lf_attn_workspace_bytes.argtypes = [C.POINTER(lf_shape)]
    lib.lf_attn_workspace_bytes.restype = C.c_size_t
    lib.lf_sparse_attn_split.argtypes = [vp, vp, vp, C.POINTER(lf_shape), C.POINTER(lf_budget), vp,
                                         C.c_float, vp, vp, C.c_size_t, vp]
    lib.lf_sparse_attn_split.restype = C.c_int
    lib.lf_sparse_attn_fwd.argtypes = [vp, vp, vp, C.POINTER(lf_shape), vp, C.c_int32, C.c_float,
                                       vp, vp, vp]
    lib.lf_sparse_attn_fwd.restype = C.c_int
    lib.lf_attn_bwd_workspace_bytes.argtypes = [C.POINTER(lf_shape)]
    lib.lf_attn_bwd_workspace_bytes.restype = C.c_size_t
    lib.lf_sparse_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, C.POINTER(lf_shape), vp, C.c_int32,
                                       C.c_float, vp, vp, vp, vp, C.c_size_t, vp]
    lib.lf_sparse_attn_bwd.restype = C.c_int
    lib.lf_qk_norm_rope.argtypes = [vp, vp, vp, vp, C.POINTER(lf_producer_shape), vp, vp]
    lib.lf_qk_norm_rope.restype = C.c_int
    lib.lf_kcache_bytes.argtypes = [C.POINTER(lf_shape), C.c_int32]
    lib.lf_kcache_bytes.restype = C.c_size_t
    lib.lf_kcache_update.argtypes = [vp, C.POINTER(lf_shape), C.c_int32, C.c_int32, C.c_int32, vp,
                                     C.c_size_t, vp]
    lib.lf_kcache_update.restype = C.c_int
    lib.lf_select_mask_cached.argtypes = [vp, vp, vp, C.c_size_t, C.c_int32, C.POINTER(lf_shape),
                                          C.POINTER(lf_budget), vp, vp, C.c_size_t, vp]
    lib.lf_select_mask_cached.restype = C.c_int
    lib.lf_init.argtypes = []
    lib.lf_init.restype = C.c_int
    lib.lf_static_scratch_bytes.argtypes = []
    lib.lf_static_scratch_bytes.restype = C.c_size_t
    lib.lf_select_mask_static.argtypes = [vp, vp, C.POINTER(lf_shape), C.POINTER(lf_budget), vp, vp]
    lib.lf_select_mask_static.restype = C.c_int
    lib.lf_strerror.argtypes = [C.c_int]
    lib.lf_strerror.restype = C.c_char_p
    lib.lf_version.argtypes = []
    lib.lf_version.restype = C.c_int
    _lib = lib
    return lib


def lf_strerror(status: int) -> str:
    return load().lf_strerror(int(status)).decode()


def lf_version() -> int:
    return int(load().lf_version())


def make_schedule(s) -> lf_schedule:
    """Build the C struct from any object with the struct's field names (e.g. synth.Schedule)."""
    out = lf_schedule()
    for name, _ in lf_schedule._fields_:
        if name != "reserved":
            setattr(out, name, getattr(s, name))
    return out


def lf_chunk_budget(chunk_idx: int, schedule) -> lf_budget:
    sch = schedule if isinstance(schedule, lf_schedule) else make_schedule(schedule)
    out = lf_budget()
    rc = load().lf_chunk_budget(int(chunk_idx), C.byref(sch), C.byref(out))
    if rc != LF_OK:
        raise LfError(rc, "lf_chunk_budget")
    return out


def make_shape(Q, K, V=None, O=None, frame_len: int = 0, block: int = 64) -> lf_shape:
    """Geometry of [H, L, d] tensors (any object with .shape and .stride() in elements)."""
    sh = lf_shape()
    sh.heads, sh.q_len, sh.head_dim = int(Q.shape[0]), int(Q.shape[1]), int(Q.shape[2])
    sh.kv_len = int(K.shape[1])
    sh.frame_len, sh.block, sh.dtype = int(frame_len), int(block), LF_BF16
    sh.q_stride_head, sh.q_stride_tok = int(Q.stride(0)), int(Q.stride(1))
    sh.k_stride_head, sh.k_stride_tok = int(K.stride(0)), int(K.stride(1))
    Vt = K if V is None else V
    Ot = Q if O is None else O
    sh.v_stride_head, sh.v_stride_tok = int(Vt.stride(0)), int(Vt.stride(1))
    sh.o_stride_head, sh.o_stride_tok = int(Ot.stride(0)), int(Ot.stride(1))
    return sh


def lf_workspace_bytes(shape: lf_shape, budget: lf_budget) -> int:
    return int(load().lf_workspace_bytes(C.byref(shape), C.byref(budget)))


def lf_workspace_layout(shape: lf_shape, budget: lf_budget) -> Tuple[int, int, int]:
    off = (C.c_size_t * 3)()
    rc = load().lf_workspace_layout(C.byref(shape), C.byref(budget), off)
    if rc != LF_OK:
        raise LfError(rc, "lf_workspace_layout")
    return int(off[0]), int(off[1]), int(off[2])


def _check_tensor(t, name: str):
    import torch
    if not t.is_cuda:
        raise ValueError(f"{name} must live in GPU memory")
    if t.dtype != torch.bfloat16:
        raise ValueError(f"{name} must be bfloat16")
    if t.dim() != 3 or t.stride(2) != 1:
        raise ValueError(f"{name} must be [H, L, d] with d contiguous")


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def lf_select_mask(Q, Kcache, frame_len: int, block: int, budget: lf_budget, indices=None,
                   workspace=None, stream=None):
    """Enqueue mask selection; returns the int32 [H, n_q, list_len] index tensor (device)."""
    import torch
    _check_tensor(Q, "Q")
    _check_tensor(Kcache, "Kcache")
    sh = make_shape(Q, Kcache, frame_len=frame_len, block=block)
    lib = load()
    need = lf_workspace_bytes(sh, budget)
    nb = -(-frame_len // block)
    n_q = (sh.q_len // frame_len) * nb if frame_len > 0 else 0
    if indices is None:
        indices = torch.empty((sh.heads, n_q, max(int(budget.list_len), 0)), dtype=torch.int32,
                              device=Q.device)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=Q.device)
    rc = lib.lf_select_mask(Q.data_ptr(), Kcache.data_ptr(), C.byref(sh), C.byref(budget),
                            indices.data_ptr(), workspace.data_ptr(),
                            workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_select_mask")
    return indices


def lf_init() -> None:
    rc = load().lf_init()
    if rc != LF_OK:
        raise LfError(rc, "lf_init")


def lf_static_scratch_bytes() -> int:
    return int(load().lf_static_scratch_bytes())


def lf_select_mask_static(Q, Kcache, frame_len: int, block: int, budget: lf_budget, indices,
                          stream=None):
    """Mask selection on the library's own static scratch; ``indices`` (int32
    [H, n_q, list_len], device) is the caller's and is returned.  Allocates nothing."""
    _check_tensor(Q, "Q")
    _check_tensor(Kcache, "Kcache")
    sh = make_shape(Q, Kcache, frame_len=frame_len, block=block)
    rc = load().lf_select_mask_static(Q.data_ptr(), Kcache.data_ptr(), C.byref(sh), C.byref(budget),
                                      indices.data_ptr(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_select_mask_static")
    return indices


def lf_kcache_bytes(shape: lf_shape, max_frames: int) -> int:
    return int(load().lf_kcache_bytes(C.byref(shape), int(max_frames)))


def lf_kcache_update(Kcache, frame_len: int, block: int, frame_begin: int, frame_end: int,
                     max_frames: int, kcache, stream=None):
    """Pool frames [frame_begin, frame_end) of Kcache into the pooled-key cache ``kcache``
    (a uint8 device tensor of >= lf_kcache_bytes())."""
    _check_tensor(Kcache, "Kcache")
    # the shape only has to describe K here: a query of one frame stands in for Q
    sh = make_shape(Kcache[:, :frame_len], Kcache, frame_len=frame_len, block=block)
    rc = load().lf_kcache_update(Kcache.data_ptr(), C.byref(sh), int(frame_begin), int(frame_end),
                                 int(max_frames), kcache.data_ptr(),
                                 kcache.numel() * kcache.element_size(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_kcache_update")


def lf_select_mask_cached(Q, kcache, max_frames: int, kv_len: int, frame_len: int, block: int,
                          budget: lf_budget, Kcache=None, indices=None, workspace=None, stream=None):
    """Mask selection with the pooled keys taken from ``kcache``; returns the index tensor.
    With ``Kcache`` the current chunk's block means are refreshed from it in the same call."""
    import torch
    _check_tensor(Q, "Q")
    if Kcache is not None:
        _check_tensor(Kcache, "Kcache")
    sh = make_shape(Q, Q if Kcache is None else Kcache, frame_len=frame_len, block=block)
    sh.kv_len = int(kv_len)
    nb = -(-frame_len // block)
    n_q = (sh.q_len // frame_len) * nb if frame_len > 0 else 0
    if indices is None:
        indices = torch.empty((sh.heads, n_q, max(int(budget.list_len), 0)), dtype=torch.int32,
                              device=Q.device)
    if workspace is None:
        workspace = torch.empty(max(lf_workspace_bytes(sh, budget), 256), dtype=torch.uint8,
                                device=Q.device)
    rc = load().lf_select_mask_cached(Q.data_ptr(), None if Kcache is None else Kcache.data_ptr(),
                                      kcache.data_ptr(),
                                      kcache.numel() * kcache.element_size(), int(max_frames),
                                      C.byref(sh), C.byref(budget), indices.data_ptr(),
                                      workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(),
                                      _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_select_mask_cached")
    return indices


def lf_sparse_attn(Q, Kcache, Vcache, indices, frame_len: int, block: int,
                   softmax_scale: float = 0.0, O=None, stream=None):
    """Enqueue blockwise sparse attention; returns O (bfloat16 [H, q_len, d], device)."""
    import torch
    _check_tensor(Q, "Q")
    _check_tensor(Kcache, "Kcache")
    _check_tensor(Vcache, "Vcache")
    if not indices.is_cuda or indices.dtype != torch.int32 or not indices.is_contiguous():
        raise ValueError("indices must be a contiguous int32 GPU tensor [H, n_q, list_len]")
    if O is None:
        O = torch.empty_like(Q, memory_format=torch.contiguous_format)
    _check_tensor(O, "O")
    sh = make_shape(Q, Kcache, Vcache, O, frame_len=frame_len, block=block)
    n_q = (sh.q_len // frame_len) * (-(-frame_len // block)) if frame_len > 0 else -1
    if indices.dim() != 3 or indices.shape[0] != sh.heads or indices.shape[1] != n_q:
        raise ValueError("indices must be [H, n_q, list_len]")
    rc = load().lf_sparse_attn(Q.data_ptr(), Kcache.data_ptr(), Vcache.data_ptr(), C.byref(sh),
                               indices.data_ptr(), int(indices.shape[-1]), float(softmax_scale),
                               O.data_ptr(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_sparse_attn")
    return O


def lf_attn_workspace_bytes(shape: lf_shape) -> int:
    return int(load().lf_attn_workspace_bytes(C.byref(shape)))


def lf_sparse_attn_split(Q, Kcache, Vcache, indices, frame_len: int, block: int, budget: lf_budget,
                         softmax_scale: float = 0.0, O=None, workspace=None, stream=None):
    """Blockwise sparse attention in two phases (dense over the current chunk, list-driven over
    the retrieved blocks); returns O.  ``indices`` as written by lf_select_mask for ``budget``."""
    import torch
    _check_tensor(Q, "Q")
    _check_tensor(Kcache, "Kcache")
    _check_tensor(Vcache, "Vcache")
    if not indices.is_cuda or indices.dtype != torch.int32 or not indices.is_contiguous():
        raise ValueError("indices must be a contiguous int32 GPU tensor [H, n_q, list_len]")
    if O is None:
        O = torch.empty_like(Q, memory_format=torch.contiguous_format)
    _check_tensor(O, "O")
    sh = make_shape(Q, Kcache, Vcache, O, frame_len=frame_len, block=block)
    n_q = (sh.q_len // frame_len) * (-(-frame_len // block)) if frame_len > 0 else -1
    if indices.dim() != 3 or tuple(indices.shape) != (sh.heads, n_q, int(budget.list_len)):
        raise ValueError("indices must be [H, n_q, budget.list_len]")
    if workspace is None:
        workspace = torch.empty(max(lf_attn_workspace_bytes(sh), 256), dtype=torch.uint8, device=Q.device)
    rc = load().lf_sparse_attn_split(Q.data_ptr(), Kcache.data_ptr(), Vcache.data_ptr(), C.byref(sh),
                                     C.byref(budget), indices.data_ptr(), float(softmax_scale),
                                     O.data_ptr(), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_sparse_attn_split")
    return O


def _check_lists(indices, sh, frame_len):
    import torch
    if not indices.is_cuda or indices.dtype != torch.int32 or not indices.is_contiguous():
        raise ValueError("indices must be a contiguous int32 GPU tensor [H, n_q, list_len]")
    n_q = (sh.q_len // frame_len) * (-(-frame_len // sh.block)) if frame_len > 0 else -1
    if indices.dim() != 3 or indices.shape[0] != sh.heads or indices.shape[1] != n_q:
        raise ValueError("indices must be [H, n_q, list_len]")


def lf_sparse_attn_fwd(Q, Kcache, Vcache, indices, frame_len: int, block: int,
                       softmax_scale: float = 0.0, O=None, lse2=None, stream=None):
    """Blockwise sparse attention that also leaves the rows' log-sum-exp (exp2 domain) for
    lf_sparse_attn_bwd; returns (O, lse2)."""
    import torch
    _check_tensor(Q, "Q")
    _check_tensor(Kcache, "Kcache")
    _check_tensor(Vcache, "Vcache")
    if O is None:
        O = torch.empty_like(Q, memory_format=torch.contiguous_format)
    _check_tensor(O, "O")
    sh = make_shape(Q, Kcache, Vcache, O, frame_len=frame_len, block=block)
    _check_lists(indices, sh, frame_len)
    if lse2 is None:
        lse2 = torch.empty((sh.heads, sh.q_len), dtype=torch.float32, device=Q.device)
    if lse2.dtype != torch.float32 or not lse2.is_cuda or not lse2.is_contiguous() \
            or tuple(lse2.shape) != (sh.heads, sh.q_len):
        raise ValueError("lse2 must be a contiguous float32 GPU tensor [H, q_len]")
    rc = load().lf_sparse_attn_fwd(Q.data_ptr(), Kcache.data_ptr(), Vcache.data_ptr(), C.byref(sh),
                                   indices.data_ptr(), int(indices.shape[-1]), float(softmax_scale),
                                   O.data_ptr(), lse2.data_ptr(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_sparse_attn_fwd")
    return O, lse2


def lf_attn_bwd_workspace_bytes(shape: lf_shape) -> int:
    return int(load().lf_attn_bwd_workspace_bytes(C.byref(shape)))


def lf_sparse_attn_bwd(Q, Kcache, Vcache, O, dO, lse2, indices, frame_len: int, block: int,
                       softmax_scale: float = 0.0, workspace=None, stream=None, grads=None):
    """Gradients of the blockwise sparse attention; returns (dQ, dK, dV), bfloat16 with the
    strides of Q, Kcache and Vcache (``grads``: three such tensors to write into instead of new
    ones).  ``indices`` ascending and duplicate-free per list."""
    import torch
    for t, name in ((Q, "Q"), (Kcache, "Kcache"), (Vcache, "Vcache"), (O, "O"), (dO, "dO")):
        _check_tensor(t, name)
    if tuple(dO.shape) != tuple(O.shape) or dO.stride() != O.stride():
        raise ValueError("dO must have the shape and strides of O")
    sh = make_shape(Q, Kcache, Vcache, O, frame_len=frame_len, block=block)
    _check_lists(indices, sh, frame_len)
    if lse2.dtype != torch.float32 or not lse2.is_cuda or not lse2.is_contiguous() \
            or tuple(lse2.shape) != (sh.heads, sh.q_len):
        raise ValueError("lse2 must be a contiguous float32 GPU tensor [H, q_len]")
    if grads is None:
        dQ = torch.empty_strided(Q.shape, Q.stride(), dtype=Q.dtype, device=Q.device)
        dK = torch.empty_strided(Kcache.shape, Kcache.stride(), dtype=Q.dtype, device=Q.device)
        dV = torch.empty_strided(Vcache.shape, Vcache.stride(), dtype=Q.dtype, device=Q.device)
    else:
        dQ, dK, dV = grads
        for g, t, name in ((dQ, Q, "dQ"), (dK, Kcache, "dK"), (dV, Vcache, "dV")):
            _check_tensor(g, name)
            if tuple(g.shape) != tuple(t.shape) or g.stride() != t.stride():
                raise ValueError(f"{name} must have the shape and strides of its input")
    if workspace is None:
        workspace = torch.empty(max(lf_attn_bwd_workspace_bytes(sh), 256), dtype=torch.uint8,
                                device=Q.device)
    rc = load().lf_sparse_attn_bwd(Q.data_ptr(), Kcache.data_ptr(), Vcache.data_ptr(), O.data_ptr(),
                                   dO.data_ptr(), lse2.data_ptr(), C.byref(sh), indices.data_ptr(),
                                   int(indices.shape[-1]), float(softmax_scale), dQ.data_ptr(),
                                   dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(),
                                   workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_sparse_attn_bwd")
    return dQ, dK, dV


def lf_qk_norm_rope(X, g, cos_table, sin_table, heads: int, Y, eps: float = 1e-6,
                    across_heads: bool = False, pairing: int = 0, stream=None):
    """RMSNorm + rotary embedding of the token-major activation X [L, >= H*d] (bfloat16) into the
    head-major tensor Y [H, L, d] (bfloat16; may be a view into Q or into the K cache)."""
    import torch
    if X.dtype != torch.bfloat16 or Y.dtype != torch.bfloat16 or X.dim() != 2 or Y.dim() != 3:
        raise ValueError("X must be bfloat16 [L, H*d] and Y bfloat16 [H, L, d]")
    if X.stride(1) != 1 or Y.stride(2) != 1 or not (X.is_cuda and Y.is_cuda):
        raise ValueError("X and Y must be GPU tensors with contiguous channels")
    for t in (g, cos_table, sin_table):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("g, cos_table, sin_table must be contiguous float32 GPU tensors")
    p = lf_producer_shape()
    p.heads, p.head_dim, p.tokens = int(heads), int(Y.shape[2]), int(X.shape[0])
    p.across_heads, p.pairing, p.eps = int(bool(across_heads)), int(pairing), float(eps)
    p.x_stride_tok, p.y_stride_tok, p.y_stride_head = int(X.stride(0)), int(Y.stride(1)), int(Y.stride(0))
    if tuple(Y.shape[:2]) != (p.heads, p.tokens) or g.numel() != p.heads * p.head_dim \
            or tuple(cos_table.shape) != (p.tokens, p.head_dim // 2) or cos_table.shape != sin_table.shape:
        raise ValueError("shapes of Y, g or the angle tables do not fit X")
    rc = load().lf_qk_norm_rope(X.data_ptr(), g.data_ptr(), cos_table.data_ptr(), sin_table.data_ptr(),
                                C.byref(p), Y.data_ptr(), _stream_ptr(stream))
    if rc != LF_OK:
        raise LfError(rc, "lf_qk_norm_rope")
    return Y
