"""ctypes binding of libdass.so -- argument marshalling only.

Function names follow the C ABI in ``include/dass.h`` (``dass_`` prefix
dropped).  Tensors are torch CUDA tensors; their ``data_ptr()`` and the current
torch stream are handed to the library, which does all the work.  There is no
fallback: if the shared library cannot be loaded the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdass.so")

DTYPE = {torch.float32: 0, torch.bfloat16: 1}
ACT = {"silu": 0, "gelu_tanh": 1, "gelu_erf": 2, "relu": 3}
AXIS = {"rows": 0, "cols": 1}

EXPORTS = (
    "dass_calib_workspace_bytes", "dass_calib_norms",
    "dass_nm_workspace_bytes", "dass_score_mask_nm",
    "dass_nm_batched_workspace_bytes", "dass_score_mask_nm_batched",
    "dass_unstructured_workspace_bytes", "dass_score_mask_unstructured", "dass_score_mask_unstructured_static",
    "dass_input_norms_workspace_bytes", "dass_input_norms",
    "dass_mlp_forward_workspace_bytes", "dass_mlp_forward", "dass_compress_24", "dass_down_proj_sparse24",
    "dass_status_string", "dass_last_error_string", "dass_version",
)


class NmTask(ctypes.Structure):
    """dass_nm_task of include/dass.h."""
    _fields_ = [("W", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("norms", ctypes.c_void_p), ("norm_axis", ctypes.c_int),
                ("group_axis", ctypes.c_int), ("alpha", ctypes.c_double), ("mask_out", ctypes.c_void_p)]


class DassError(RuntimeError):
    """A libdass call returned a status other than DASS_OK."""

    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name}: {detail}" if detail else name)
        self.status = status
        self.status_name = name


_lib = None


def library_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libdass.so.  A library that is missing, or was built from other sources than the
    present ones (compared by content hash), is rebuilt with hipcc first; if that fails the
    call raises: a binary older than its sources is never used."""
    global _lib
    if _lib is not None:
        return _lib
    from . import build as _build
    if _build.is_stale():
        _build.build()
    lib = ctypes.CDLL(_LIB_PATH)
    i64, sz, vp, ci, dbl = (ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_int,
                            ctypes.c_double)
    lib.dass_calib_workspace_bytes.restype = sz
    lib.dass_calib_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.dass_calib_norms.restype = ci
    lib.dass_calib_norms.argtypes = [vp, i64, i64, vp, vp, i64, i64, i64, ci, ci, vp, ci, vp,
                                     vp, sz, vp]
    lib.dass_nm_workspace_bytes.restype = sz
    lib.dass_nm_workspace_bytes.argtypes = [i64, i64, ci]
    lib.dass_score_mask_nm.restype = ci
    lib.dass_score_mask_nm.argtypes = [vp, i64, i64, i64, ci, vp, ci, ci, dbl, ci, ci, vp,
                                       vp, sz, vp]
    lib.dass_nm_batched_workspace_bytes.restype = sz
    lib.dass_nm_batched_workspace_bytes.argtypes = [ctypes.POINTER(NmTask), i64]
    lib.dass_score_mask_nm_batched.restype = ci
    lib.dass_score_mask_nm_batched.argtypes = [ctypes.POINTER(NmTask), i64, ci, ci, ci, vp, sz, vp]
    lib.dass_unstructured_workspace_bytes.restype = sz
    lib.dass_unstructured_workspace_bytes.argtypes = [i64, i64, ci, ci, ci]
    lib.dass_score_mask_unstructured.restype = ci
    lib.dass_score_mask_unstructured.argtypes = [vp, i64, i64, i64, ci, vp, ci, ci, dbl, i64, vp,
                                                 vp, sz, vp]
    lib.dass_score_mask_unstructured_static.restype = ci
    lib.dass_score_mask_unstructured_static.argtypes = [vp, i64, i64, i64, ci, vp, ci, ci, dbl, i64, vp, vp]
    lib.dass_input_norms_workspace_bytes.restype = sz
    lib.dass_input_norms_workspace_bytes.argtypes = [i64, i64]
    lib.dass_input_norms.restype = ci
    lib.dass_input_norms.argtypes = [vp, i64, i64, i64, ci, vp, ci, vp, vp, sz, vp]
    lib.dass_mlp_forward_workspace_bytes.restype = sz
    lib.dass_mlp_forward_workspace_bytes.argtypes = [i64, i64, i64, ci]
    lib.dass_mlp_forward.restype = ci
    lib.dass_mlp_forward.argtypes = [vp, i64, i64, vp, vp, i64, vp, i64, i64, i64, ci, ci, vp, i64,
                                     vp, sz, vp]
    lib.dass_compress_24.restype = ci
    lib.dass_compress_24.argtypes = [vp, i64, i64, i64, ci, ci, vp, i64, vp, i64, vp, vp]
    lib.dass_down_proj_sparse24.restype = ci
    lib.dass_down_proj_sparse24.argtypes = [vp, i64, i64, vp, i64, vp, i64, i64, i64, ci, vp, i64, vp]
    lib.dass_status_string.restype = ctypes.c_char_p
    lib.dass_status_string.argtypes = [ci]
    lib.dass_last_error_string.restype = ctypes.c_char_p
    lib.dass_last_error_string.argtypes = []
    lib.dass_version.restype = ci
    lib.dass_version.argtypes = []
    _lib = lib
    return lib


def version() -> int:
    return int(load_library().dass_version())


def _check(status: int) -> None:
    if status != 0:
        lib = load_library()
        raise DassError(status, lib.dass_status_string(status).decode(),
                        lib.dass_last_error_string().decode())


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _matrix(t: torch.Tensor, name: str):
    if t.dim() != 2 or t.stride(1) != 1 or t.dtype not in DTYPE:
        raise TypeError(f"{name}: need a 2-D f32/bf16 tensor with unit column stride")
    return t.shape[0], t.shape[1], t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1])


def _scratch(nbytes: int, device, stream=None) -> torch.Tensor:
    """A workspace for a caller that passed none.  This is a convenience of the binding (the
    library itself never allocates): the block comes from torch's caching allocator and is
    released when the call returns, so it is tied to the stream the kernels run on; a caller
    that wants no allocation on its path passes ``workspace`` itself."""
    buf = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    if stream is not None:
        buf.record_stream(stream)   # the allocator may not hand the block on before `stream` is done with it
    return buf


# ------------------------------------------------------------------ stage 1 --
def calib_workspace_bytes(T: int, d: int, d_int: int, dtype: torch.dtype) -> int:
    return int(load_library().dass_calib_workspace_bytes(T, d, d_int, DTYPE[dtype]))


def calib_norms(X: torch.Tensor, Wgate: torch.Tensor, Wup: torch.Tensor, act: str,
                sumsq: torch.Tensor, accumulate: bool = False,
                norms_out: Optional[torch.Tensor] = None,
                workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """dass_calib_norms: sumsq (+)= sum_t y[t, :]^2 with y = act(X Wgate^T) * (X Wup^T)."""
    lib = load_library()
    T, d, ldx = _matrix(X, "X")
    d_int, dg, ldw = _matrix(Wgate, "Wgate")
    d_int_u, du, ldw_u = _matrix(Wup, "Wup")
    if (d_int_u, du, ldw_u) != (d_int, dg, ldw) or dg != d or not (X.dtype == Wgate.dtype == Wup.dtype):
        raise ValueError("X, Wgate, Wup disagree in shape, stride or dtype")
    if sumsq.dtype != torch.float32 or sumsq.numel() != d_int or not sumsq.is_contiguous():
        raise TypeError("sumsq: need contiguous float32[d_int]")
    if norms_out is not None and (norms_out.dtype != torch.float32 or norms_out.numel() != d_int
                                  or not norms_out.is_contiguous()):
        raise TypeError("norms_out: need contiguous float32[d_int]")
    need = int(lib.dass_calib_workspace_bytes(T, d, d_int, DTYPE[X.dtype]))
    if workspace is None and need > 0:
        workspace = _scratch(need, X.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.dass_calib_norms(_ptr(X), T, ldx, _ptr(Wgate), _ptr(Wup), ldw, d, d_int,
                                DTYPE[X.dtype], ACT[act], _ptr(sumsq), int(bool(accumulate)),
                                _ptr(norms_out), _ptr(workspace), ws_bytes, _stream(stream)))


def input_norms_workspace_bytes(T: int, d: int) -> int:
    return int(load_library().dass_input_norms_workspace_bytes(T, d))


def input_norms(X: torch.Tensor, sumsq: torch.Tensor, accumulate: bool = False,
                norms_out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                stream=None) -> None:
    """dass_input_norms: sumsq[j] (+)= sum_t X[t, j]^2 (the Wanda metric's input norms, Eq. 1)."""
    lib = load_library()
    T, d, ldx = _matrix(X, "X")
    for name, t in (("sumsq", sumsq), ("norms_out", norms_out)):
        if t is not None and (t.dtype != torch.float32 or t.numel() != d or not t.is_contiguous()):
            raise TypeError(f"{name}: need contiguous float32[d]")
    if workspace is None:
        workspace = _scratch(int(lib.dass_input_norms_workspace_bytes(T, d)), X.device, stream)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.dass_input_norms(_ptr(X), T, ldx, d, DTYPE[X.dtype], _ptr(sumsq), int(bool(accumulate)),
                                _ptr(norms_out), _ptr(workspace), ws_bytes, _stream(stream)))


def mlp_forward_workspace_bytes(T: int, d: int, d_int: int, dtype=torch.bfloat16) -> int:
    return int(load_library().dass_mlp_forward_workspace_bytes(T, d, d_int, DTYPE[dtype]))


def mlp_forward(X: torch.Tensor, Wgate: torch.Tensor, Wup: torch.Tensor, Wdown: Optional[torch.Tensor], act: str,
                out: Optional[torch.Tensor], workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """dass_mlp_forward: out = (act(X Wgate^T) * (X Wup^T)) Wdown^T (Eq. 2 then Eq. 3).

    With ``Wdown=None`` only Eq. 2 runs: y is left in ``workspace`` (required then) as [T, d_int].
    """
    lib = load_library()
    T, d, ldx = _matrix(X, "X")
    d_int, d2, ldw = _matrix(Wgate, "Wgate")
    if _matrix(Wup, "Wup") != (d_int, d2, ldw) or d2 != d:
        raise ValueError("Wgate and Wup must be [d_int, d] with one leading dimension")
    ldd = ldo = 0
    if Wdown is None:
        if workspace is None:
            raise ValueError("Wdown=None leaves y in the workspace: pass one")
        out = None
        dtypes = {X.dtype, Wgate.dtype, Wup.dtype}
    else:
        dd, di, ldd = _matrix(Wdown, "Wdown")
        To, do, ldo = _matrix(out, "out")
        if (dd, di) != (d, d_int) or (To, do) != (T, d):
            raise ValueError("Wdown must be [d, d_int] and out [T, d]")
        dtypes = {X.dtype, Wgate.dtype, Wup.dtype, Wdown.dtype, out.dtype}
    if len(dtypes) != 1:
        raise TypeError("X, the weights and out must share one dtype")
    if workspace is None:
        workspace = _scratch(int(lib.dass_mlp_forward_workspace_bytes(T, d, d_int, DTYPE[X.dtype])), X.device, stream)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib.dass_mlp_forward(_ptr(X), T, ldx, _ptr(Wgate), _ptr(Wup), ldw, _ptr(Wdown), ldd, d, d_int,
                                DTYPE[X.dtype], ACT[act], _ptr(out), ldo, _ptr(workspace), ws_bytes,
                                _stream(stream)))


# ------------------------------------------------------------------ stage 2 --
def nm_workspace_bytes(rows: int, cols: int, norm_axis: str) -> int:
    return int(load_library().dass_nm_workspace_bytes(rows, cols, AXIS[norm_axis]))


def score_mask_nm(W: torch.Tensor, norms: torch.Tensor, norm_axis: str, group_axis: str,
                  alpha: float, n_keep: int, m: int, mask_out: Optional[torch.Tensor] = None,
                  workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """dass_score_mask_nm: in-place N:M pruning of W by |W| * norms^alpha."""
    lib = load_library()
    rows, cols, ld = _matrix(W, "W")
    if norms.dtype != torch.float32 or not norms.is_contiguous():
        raise TypeError("norms: need contiguous float32")
    if norms.numel() != (rows if norm_axis == "rows" else cols):
        raise ValueError("norms length does not match norm_axis")
    if mask_out is not None and (mask_out.dtype != torch.uint8 or not mask_out.is_contiguous()
                                 or mask_out.numel() != rows * (cols // 8)):
        raise TypeError("mask_out: need contiguous uint8[rows * cols / 8]")
    need = int(lib.dass_nm_workspace_bytes(rows, cols, AXIS[norm_axis]))
    if workspace is None:
        workspace = _scratch(need, W.device, stream)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.dass_score_mask_nm(_ptr(W), rows, cols, ld, DTYPE[W.dtype], _ptr(norms),
                                  AXIS[norm_axis], AXIS[group_axis], float(alpha), int(n_keep),
                                  int(m), _ptr(mask_out), _ptr(workspace), ws_bytes,
                                  _stream(stream)))


def _nm_task_array(tasks):
    """tasks: sequence of (W, norms, norm_axis, group_axis, alpha[, mask_out]) -> (NmTask array, dtype, device)."""
    arr = (NmTask * max(len(tasks), 1))()
    dtype = device = None
    for i, t in enumerate(tasks):
        W, norms, norm_axis, group_axis, alpha = t[:5]
        mask_out = t[5] if len(t) > 5 else None
        rows, cols, ld = _matrix(W, f"tasks[{i}].W")
        if dtype is None:
            dtype, device = W.dtype, W.device
        elif W.dtype != dtype:
            raise TypeError("all matrices of a batched call must share one dtype")
        if norms.dtype != torch.float32 or not norms.is_contiguous():
            raise TypeError(f"tasks[{i}].norms: need contiguous float32")
        if norms.numel() != (rows if norm_axis == "rows" else cols):
            raise ValueError(f"tasks[{i}]: norms length does not match norm_axis")
        if mask_out is not None and (mask_out.dtype != torch.uint8 or not mask_out.is_contiguous()
                                     or mask_out.numel() != rows * (cols // 8)):
            raise TypeError(f"tasks[{i}].mask_out: need contiguous uint8[rows * cols / 8]")
        arr[i] = NmTask(W.data_ptr(), rows, cols, ld, norms.data_ptr(), AXIS[norm_axis], AXIS[group_axis],
                        float(alpha), None if mask_out is None else mask_out.data_ptr())
    return arr, dtype, device


def nm_batched_workspace_bytes(tasks) -> int:
    arr, _, _ = _nm_task_array(tasks)
    return int(load_library().dass_nm_batched_workspace_bytes(arr, len(tasks)))


def score_mask_nm_batched(tasks, n_keep: int, m: int, workspace: Optional[torch.Tensor] = None,
                          stream=None) -> None:
    """dass_score_mask_nm_batched: score_mask_nm over many matrices, equal ones sharing launches.

    tasks: sequence of (W, norms, norm_axis, group_axis, alpha[, mask_out]).
    """
    lib = load_library()
    if len(tasks) == 0:
        return
    arr, dtype, device = _nm_task_array(tasks)
    if workspace is None:
        workspace = _scratch(int(lib.dass_nm_batched_workspace_bytes(arr, len(tasks))), device, stream)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.dass_score_mask_nm_batched(arr, len(tasks), DTYPE[dtype], int(n_keep), int(m),
                                          _ptr(workspace), ws_bytes, _stream(stream)))


def unstructured_workspace_bytes(rows: int, cols: int, dtype: torch.dtype, norm_axis: str,
                                 group_axis: str) -> int:
    return int(load_library().dass_unstructured_workspace_bytes(
        rows, cols, DTYPE[dtype], AXIS[norm_axis], AXIS[group_axis]))


def score_mask_unstructured(W: torch.Tensor, norms: torch.Tensor, norm_axis: str, group_axis: str,
                            alpha: float, n_prune: int, mask_out: Optional[torch.Tensor] = None,
                            workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    """dass_score_mask_unstructured: prune the n_prune lowest scores of every line."""
    lib = load_library()
    rows, cols, ld = _matrix(W, "W")
    if norms.dtype != torch.float32 or not norms.is_contiguous():
        raise TypeError("norms: need contiguous float32")
    if norms.numel() != (rows if norm_axis == "rows" else cols):
        raise ValueError("norms length does not match norm_axis")
    if mask_out is not None and (mask_out.dtype != torch.uint8 or not mask_out.is_contiguous()
                                 or mask_out.numel() != rows * (cols // 8)):
        raise TypeError("mask_out: need contiguous uint8[rows * cols / 8]")
    need = int(lib.dass_unstructured_workspace_bytes(rows, cols, DTYPE[W.dtype], AXIS[norm_axis],
                                                     AXIS[group_axis]))
    if workspace is None:
        workspace = _scratch(need, W.device, stream)
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.dass_score_mask_unstructured(_ptr(W), rows, cols, ld, DTYPE[W.dtype], _ptr(norms),
                                            AXIS[norm_axis], AXIS[group_axis], float(alpha),
                                            int(n_prune), _ptr(mask_out), _ptr(workspace), ws_bytes,
                                            _stream(stream)))


def score_mask_unstructured_static(W: torch.Tensor, norms: torch.Tensor, norm_axis: str, group_axis: str,
                                   alpha: float, n_prune: int, mask_out: Optional[torch.Tensor] = None,
                                   stream=None) -> None:
    """dass_score_mask_unstructured_static: the same selection with the library's own device scratch."""
    lib = load_library()
    rows, cols, ld = _matrix(W, "W")
    if norms.dtype != torch.float32 or not norms.is_contiguous():
        raise TypeError("norms: need contiguous float32")
    if norms.numel() != (rows if norm_axis == "rows" else cols):
        raise ValueError("norms length does not match norm_axis")
    if mask_out is not None and (mask_out.dtype != torch.uint8 or not mask_out.is_contiguous()
                                 or mask_out.numel() != rows * (cols // 8)):
        raise TypeError("mask_out: need contiguous uint8[rows * cols / 8]")
    _check(lib.dass_score_mask_unstructured_static(_ptr(W), rows, cols, ld, DTYPE[W.dtype], _ptr(norms),
                                                   AXIS[norm_axis], AXIS[group_axis], float(alpha),
                                                   int(n_prune), _ptr(mask_out), _stream(stream)))


def compress_24(W: torch.Tensor, group_axis: str, values_out: torch.Tensor, meta_out: torch.Tensor,
                surplus_out: Optional[torch.Tensor] = None, stream=None) -> None:
    """dass_compress_24: kept values and 2-bit position codes of a 2:4 sparse matrix."""
    lib = load_library()
    rows, cols, ld = _matrix(W, "W")
    vr, vc, ldv = _matrix(values_out, "values_out")
    if values_out.dtype != W.dtype or (vr, vc) != ((rows // 2, cols) if group_axis == "rows" else (rows, cols // 2)):
        raise TypeError("values_out: need W's dtype and [rows / 2, cols] (rows) or [rows, cols / 2] (cols)")
    want = (rows // 4, cols // 2) if group_axis == "rows" else (rows, cols // 8)
    if meta_out.dtype != torch.uint8 or meta_out.dim() != 2 or tuple(meta_out.shape) != want or meta_out.stride(1) != 1:
        raise TypeError(f"meta_out: need uint8 {want}")
    ldm = meta_out.stride(0) if meta_out.shape[0] > 1 else max(meta_out.stride(0), meta_out.shape[1])
    if surplus_out is not None and (surplus_out.dtype != torch.int64 or surplus_out.numel() != 1):
        raise TypeError("surplus_out: need one int64")
    _check(lib.dass_compress_24(_ptr(W), rows, cols, ld, DTYPE[W.dtype], AXIS[group_axis], _ptr(values_out), ldv,
                                _ptr(meta_out), ldm, _ptr(surplus_out), _stream(stream)))


def down_proj_sparse24(Y: torch.Tensor, values: torch.Tensor, meta: torch.Tensor, out: torch.Tensor,
                       stream=None) -> None:
    """dass_down_proj_sparse24: out = Y Wdown^T from the 2:4 compressed Down-Proj (sparse MFMA)."""
    lib = load_library()
    T, d_int, ldy = _matrix(Y, "Y")
    d, half, ldv = _matrix(values, "values")
    To, do, ldo = _matrix(out, "out")
    if half * 2 != d_int or (To, do) != (T, d) or values.dtype != Y.dtype or out.dtype != Y.dtype:
        raise ValueError("need values [d, d_int / 2] and out [T, d] in Y's dtype")
    if meta.dtype != torch.uint8 or meta.dim() != 2 or tuple(meta.shape) != (d, d_int // 8) or meta.stride(1) != 1:
        raise TypeError("meta: need uint8 [d, d_int / 8]")
    ldm = meta.stride(0) if meta.shape[0] > 1 else max(meta.stride(0), meta.shape[1])
    _check(lib.dass_down_proj_sparse24(_ptr(Y), T, ldy, _ptr(values), ldv, _ptr(meta), ldm, d, d_int,
                                       DTYPE[Y.dtype], _ptr(out), ldo, _stream(stream)))

