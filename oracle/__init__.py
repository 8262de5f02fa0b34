"""Float64 CPU oracle for the DaSS hot path -- TEST INFRASTRUCTURE ONLY.

Thin ctypes access to ``dass_oracle.c`` (plain C, double arithmetic).  The GPU
library and its Python binding never import this package; only the tests, the
smoke check and the benchmark's CPU-baseline leg do.  Inputs are numpy float32
arrays holding exactly the values the GPU is given (bf16 widens to float32
without rounding).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dass_oracle.c")
_LIB = os.path.join(_HERE, "libdass_oracle.so")

ACT = {"silu": 0, "gelu_tanh": 1, "gelu_erf": 2, "relu": 3}
AXIS = {"rows": 0, "cols": 1}


def build(force: bool = False) -> str:
    """Compile dass_oracle.c with gcc (OpenMP) into libdass_oracle.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=gnu11",
               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        # DASS_ORACLE_LIB: another build of dass_oracle.c to load instead (the sanitizer test's)
        path = os.environ.get("DASS_ORACLE_LIB") or build()
        lib = ctypes.CDLL(path)
        i64, dbl, vp, ci = ctypes.c_int64, ctypes.c_double, ctypes.c_void_p, ctypes.c_int
        lib.oracle_act.restype = dbl
        lib.oracle_act.argtypes = [dbl, ci]
        lib.oracle_sumsq.restype = None
        lib.oracle_sumsq.argtypes = [vp, i64, i64, vp, vp, i64, i64, i64, ci, vp, i64, vp]
        lib.oracle_input_sumsq.restype = None
        lib.oracle_input_sumsq.argtypes = [vp, i64, i64, i64, vp]
        lib.oracle_norms.restype = None
        lib.oracle_norms.argtypes = [vp, i64, vp]
        lib.oracle_factor.restype = None
        lib.oracle_factor.argtypes = [vp, i64, dbl, vp]
        lib.oracle_mask_nm.restype = ci
        lib.oracle_mask_nm.argtypes = [vp, i64, i64, i64, vp, ci, ci, ci, ci, vp]
        lib.oracle_mask_unstructured.restype = ci
        lib.oracle_mask_unstructured.argtypes = [vp, i64, i64, i64, vp, ci, ci, i64, vp]
        lib.oracle_mlp_forward.restype = None
        lib.oracle_mlp_forward.argtypes = [vp, i64, i64, vp, vp, i64, vp, i64, i64, i64, ci, vp, i64, vp, vp]
        lib.oracle_compress_24.restype = i64
        lib.oracle_compress_24.argtypes = [vp, i64, i64, i64, ci, vp, i64, vp, i64]
        lib.oracle_down_sparse24.restype = None
        lib.oracle_down_sparse24.argtypes = [vp, i64, i64, vp, i64, vp, i64, i64, i64, vp, i64, vp, vp]
        lib.oracle_num_threads.restype = ci
        lib.oracle_num_threads.argtypes = []
        _lib = lib
    return _lib


def _f32_2d(a, name):
    a = np.asarray(a)
    if a.dtype != np.float32 or a.ndim != 2:
        raise TypeError(f"{name}: need a 2-D float32 array")
    if (a.shape[1] > 1 and a.strides[1] != 4) or (a.shape[0] > 1 and a.strides[0] % 4 != 0):
        raise TypeError(f"{name}: need unit column stride")
    return a


def _ld(a):
    """Row stride in elements (any value serves when there is a single row)."""
    return a.strides[0] // 4 if a.shape[0] > 1 else a.shape[1]


def _own_copy(W):
    W = np.asarray(W)
    if W.dtype != np.float32 or W.ndim != 2:
        raise TypeError("W: need a 2-D float32 array")
    return np.array(W, dtype=np.float32, order="C", copy=True)


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def act(g: float, kind: str) -> float:
    """sigma(g) of Eq. 2 for one of 'silu', 'gelu_tanh', 'gelu_erf', 'relu'."""
    return float(_load().oracle_act(float(g), ACT[kind]))


def sumsq(X, Wg, Wu, kind: str, neurons=None, out=None) -> np.ndarray:
    """Add sum_t (sigma(x_t.Wg_i) * (x_t.Wu_i))^2 into ``out`` (float64) and return it.

    ``neurons`` restricts the computation to the listed rows of Wg/Wu; ``out``
    then has one entry per listed neuron.  Passing the previous result as
    ``out`` accumulates over token chunks.
    """
    X, Wg, Wu = _f32_2d(X, "X"), _f32_2d(Wg, "Wg"), _f32_2d(Wu, "Wu")
    T, d = X.shape
    d_int = Wg.shape[0]
    if Wg.shape != Wu.shape or Wg.shape[1] != d or _ld(Wg) != _ld(Wu):
        raise ValueError("shape mismatch between X, Wg, Wu")
    if neurons is not None:
        neurons = np.ascontiguousarray(neurons, dtype=np.int64)
        if neurons.size and (neurons.min() < 0 or neurons.max() >= d_int):
            raise ValueError("neuron index out of range")
    n = d_int if neurons is None else neurons.size
    if out is None:
        out = np.zeros(n, dtype=np.float64)
    if out.dtype != np.float64 or out.shape != (n,) or not out.flags.c_contiguous:
        raise TypeError("out: need contiguous float64 of matching length")
    _load().oracle_sumsq(_ptr(X), T, _ld(X), _ptr(Wg), _ptr(Wu), _ld(Wg),
                         d, d_int, ACT[kind],
                         None if neurons is None else _ptr(neurons), n, _ptr(out))
    return out


def input_sumsq(X, out=None) -> np.ndarray:
    """Add sum_t X[t, j]^2 (Eq. 1: the squared input-feature norms) into ``out`` (float64)."""
    X = _f32_2d(X, "X")
    T, d = X.shape
    if out is None:
        out = np.zeros(d, dtype=np.float64)
    if out.dtype != np.float64 or out.shape != (d,) or not out.flags.c_contiguous:
        raise TypeError("out: need contiguous float64 of length d")
    _load().oracle_input_sumsq(_ptr(X), T, _ld(X), d, _ptr(out))
    return out


def norms(sumsq_vec) -> np.ndarray:
    """||y_i||_2 = sqrt(sumsq_i), float64."""
    s = np.ascontiguousarray(sumsq_vec, dtype=np.float64)
    out = np.empty_like(s)
    _load().oracle_norms(_ptr(s), s.size, _ptr(out))
    return out


def factor(norms32, alpha: float) -> np.ndarray:
    """f = (float) norm^alpha from float32 norms (Eq. 4 / Eq. 5)."""
    n = np.ascontiguousarray(norms32)
    if n.dtype != np.float32 or n.ndim != 1:
        raise TypeError("norms32: need 1-D float32")
    out = np.empty_like(n)
    _load().oracle_factor(_ptr(n), n.size, float(alpha), _ptr(out))
    return out


def _mask_buf(rows, cols, want):
    if not want:
        return None
    return np.zeros((rows, (cols + 7) // 8), dtype=np.uint8)


def mask_nm(W, norms32, norm_axis: str, group_axis: str, alpha: float, n_keep: int, m: int,
            want_mask: bool = False):
    """N:M selection on scores |W| * norm^alpha; returns (pruned copy of W, packed mask or None)."""
    W = _own_copy(W)
    rows, cols = W.shape
    f = factor(norms32, alpha)
    if f.size != (rows if norm_axis == "rows" else cols):
        raise ValueError("norms length does not match norm_axis")
    mask = _mask_buf(rows, cols, want_mask)
    rc = _load().oracle_mask_nm(_ptr(W), rows, cols, cols, _ptr(f),
                                AXIS[norm_axis], AXIS[group_axis], int(n_keep), int(m),
                                None if mask is None else _ptr(mask))
    if rc != 0:
        raise ValueError("oracle_mask_nm rejected the arguments")
    return W, mask


def mask_unstructured(W, norms32, norm_axis: str, group_axis: str, alpha: float, n_prune: int,
                      want_mask: bool = False):
    """Per-line unstructured selection; returns (pruned copy of W, packed mask or None)."""
    W = _own_copy(W)
    rows, cols = W.shape
    f = factor(norms32, alpha)
    if f.size != (rows if norm_axis == "rows" else cols):
        raise ValueError("norms length does not match norm_axis")
    mask = _mask_buf(rows, cols, want_mask)
    rc = _load().oracle_mask_unstructured(_ptr(W), rows, cols, cols, _ptr(f),
                                          AXIS[norm_axis], AXIS[group_axis], int(n_prune),
                                          None if mask is None else _ptr(mask))
    if rc != 0:
        raise ValueError("oracle_mask_unstructured rejected the arguments")
    return W, mask


def mlp_forward(X, Wg, Wu, Wd, kind: str, tokens=None, want_abs: bool = False):
    """Eq. 2 then Eq. 3 in float64: out[t, :] = (sigma(x_t Wg^T) * (x_t Wu^T)) Wd^T.

    ``tokens`` restricts the computation to the listed rows of X.  With ``want_abs`` also returns
    sum_i |y_i Wd[j, i]| per output, the scale of the sum's rounding error.
    """
    X, Wg, Wu, Wd = _f32_2d(X, "X"), _f32_2d(Wg, "Wg"), _f32_2d(Wu, "Wu"), _f32_2d(Wd, "Wd")
    T, d = X.shape
    d_int = Wg.shape[0]
    if Wg.shape != Wu.shape or Wg.shape[1] != d or _ld(Wg) != _ld(Wu) or Wd.shape != (d, d_int):
        raise ValueError("shape mismatch between X, Wg, Wu, Wd")
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int64)
        if tokens.size and (tokens.min() < 0 or tokens.max() >= T):
            raise ValueError("token index out of range")
    n = T if tokens is None else tokens.size
    out = np.empty((n, d), dtype=np.float64)
    absout = np.empty((n, d), dtype=np.float64) if want_abs else None
    _load().oracle_mlp_forward(_ptr(X), T, _ld(X), _ptr(Wg), _ptr(Wu), _ld(Wg), _ptr(Wd), _ld(Wd),
                               d, d_int, ACT[kind], None if tokens is None else _ptr(tokens), n,
                               _ptr(out), None if absout is None else _ptr(absout))
    return (out, absout) if want_abs else out


def compress_24(W, group_axis: str):
    """2:4 compressed form of W along ``group_axis``: (values float32, meta uint8, surplus groups).

    values is [rows, cols/2] (cols) or [rows/2, cols] (rows); meta holds one nibble p0 | p1 << 2
    per group, [rows, cols/8] or [rows/4, ceil(cols/2)].
    """
    W = _f32_2d(W, "W")
    rows, cols = W.shape
    if group_axis == "cols":
        values = np.zeros((rows, cols // 2), dtype=np.float32)
        meta = np.zeros((rows, cols // 8), dtype=np.uint8)
    else:
        values = np.zeros((rows // 2, cols), dtype=np.float32)
        meta = np.zeros((rows // 4, (cols + 1) // 2), dtype=np.uint8)
    rc = _load().oracle_compress_24(_ptr(W), rows, cols, _ld(W), AXIS[group_axis],
                                    _ptr(values), values.shape[1], _ptr(meta), meta.shape[1])
    if rc < 0:
        raise ValueError("oracle_compress_24 rejected the shape")
    return values, meta, int(rc)


def down_sparse24(Y, values, meta, tokens=None, want_abs: bool = False):
    """Eq. 3 from the 2:4 compressed Down-Proj (groups along the columns): out = Y W^T in float64."""
    Y, values = _f32_2d(Y, "Y"), _f32_2d(values, "values")
    meta = np.asarray(meta)
    T, d_int = Y.shape
    d = values.shape[0]
    if meta.dtype != np.uint8 or meta.ndim != 2 or not meta.flags.c_contiguous:
        raise TypeError("meta: need a contiguous 2-D uint8 array")
    if d_int % 8 != 0 or values.shape != (d, d_int // 2) or meta.shape != (d, d_int // 8):
        raise ValueError("shape mismatch between Y, values and meta")
    if tokens is not None:
        tokens = np.ascontiguousarray(tokens, dtype=np.int64)
        if tokens.size and (tokens.min() < 0 or tokens.max() >= T):
            raise ValueError("token index out of range")
    n = T if tokens is None else tokens.size
    out = np.empty((n, d), dtype=np.float64)
    absout = np.empty((n, d), dtype=np.float64) if want_abs else None
    _load().oracle_down_sparse24(_ptr(Y), T, _ld(Y), _ptr(values), _ld(values), _ptr(meta), meta.shape[1], d, d_int,
                                 None if tokens is None else _ptr(tokens), n, _ptr(out),
                                 None if absout is None else _ptr(absout))
    return (out, absout) if want_abs else out
