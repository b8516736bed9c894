"""CPU oracle (test infrastructure only).

Nothing in the product package imports this.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` do.

* ``oracle.c``        - SpMM / SDDMM / edge-softmax by their plain definitions,
                        double accumulation, CSR order (paper Section 2.2,
                        Eq. 2 and Eq. 4 for what each operator touches).
* ``planner_ref.py``  - the workload-distribution and load-balancing steps of
                        Sections 4.2-4.3 in plain Python, used to check the
                        product planner's output bit for bit.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

F16, BF16, F32 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile oracle.c with gcc (OpenMP over rows, for timing only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_half_to_double.restype = ctypes.c_double
        _lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        _lib.oracle_bf16_to_double.restype = ctypes.c_double
        _lib.oracle_bf16_to_double.argtypes = [ctypes.c_uint16]
        _lib.oracle_max_threads.restype = ctypes.c_int
    return _lib


def _p(a):
    return None if a is None else ctypes.c_void_p(a.ctypes.data)


def _dt(a: np.ndarray, bf16: bool = False) -> int:
    if bf16:
        assert a.dtype == np.uint16
        return BF16
    if a.dtype == np.float16:
        return F16
    if a.dtype == np.float32:
        return F32
    raise TypeError(f"unsupported dtype {a.dtype}")


def max_threads() -> int:
    return int(lib().oracle_max_threads())


def half_to_double(bits: int) -> float:
    return float(lib().oracle_half_to_double(ctypes.c_uint16(bits)))


def bf16_to_double(bits: int) -> float:
    return float(lib().oracle_bf16_to_double(ctypes.c_uint16(bits)))


def widen(a: np.ndarray, bf16: bool = False) -> np.ndarray:
    a = np.ascontiguousarray(a)
    out = np.empty(a.size, dtype=np.float64)
    lib().oracle_widen(_p(a), ctypes.c_int(_dt(a, bf16)), ctypes.c_int64(a.size), _p(out))
    return out.reshape(a.shape)


def spmm(rowptr, col, val, B, rows=None, nthreads: int = 0, want_scale: bool = True,
         bf16: bool = False):
    """C = A @ B (double).  ``rows``: optional int64 list of rows to compute.
    Returns (C, S) with S = |A| @ |B| (or None)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val)
    B = np.ascontiguousarray(B)
    M = rowptr.size - 1
    N = B.shape[1]
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
    R = M if rows is None else rows.size
    C = np.empty((R, N), dtype=np.float64)
    S = np.empty((R, N), dtype=np.float64) if want_scale else None
    rc = lib().oracle_spmm(ctypes.c_int64(M), _p(rowptr), _p(col), _p(val), ctypes.c_int(_dt(val, bf16)),
                           _p(B), ctypes.c_int(_dt(B, bf16)), ctypes.c_int64(N), ctypes.c_int64(N),
                           _p(rows), ctypes.c_int64(R), _p(C), _p(S), ctypes.c_int(nthreads))
    if rc != 0:
        raise RuntimeError(f"oracle_spmm failed: {rc}")
    return C, S


def sddmm(rowptr, col, val, X, Y, idx=None, nthreads: int = 0, want_scale: bool = True,
          bf16: bool = False):
    """out[p] = val[p] * <X[row(p)], Y[col[p]]> (double), CSR order, or only at
    the CSR positions ``idx``.  Returns (out, S)."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val)
    X = np.ascontiguousarray(X)
    Y = np.ascontiguousarray(Y)
    assert X.dtype == Y.dtype and X.shape[1] == Y.shape[1]
    M = rowptr.size - 1
    K = X.shape[1]
    if idx is None:
        n = int(rowptr[-1])
        idx_row = None
    else:
        idx = np.ascontiguousarray(idx, dtype=np.int64)
        idx_row = (np.searchsorted(rowptr, idx, side="right") - 1).astype(np.int64)
        n = idx.size
    out = np.empty(n, dtype=np.float64)
    S = np.empty(n, dtype=np.float64) if want_scale else None
    rc = lib().oracle_sddmm(ctypes.c_int64(M), _p(rowptr), _p(col), _p(val), ctypes.c_int(_dt(val, bf16)),
                            _p(X), _p(Y), ctypes.c_int(_dt(X, bf16)), ctypes.c_int64(K),
                            _p(idx), _p(idx_row), ctypes.c_int64(n), _p(out), _p(S), ctypes.c_int(nthreads))
    if rc != 0:
        raise RuntimeError(f"oracle_sddmm failed: {rc}")
    return out, S


def edge_softmax(rowptr, scores, scale: float = 1.0, nthreads: int = 0) -> np.ndarray:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    scores = np.ascontiguousarray(scores, dtype=np.float64)
    M = rowptr.size - 1
    alpha = np.zeros(scores.size, dtype=np.float64)
    rc = lib().oracle_edge_softmax(ctypes.c_int64(M), _p(rowptr), _p(scores), ctypes.c_double(scale),
                                   _p(alpha), ctypes.c_int(nthreads))
    if rc != 0:
        raise RuntimeError(f"oracle_edge_softmax failed: {rc}")
    return alpha


def attention_head(rowptr, col, val, X, Y, B, scale: float, nthreads: int = 0):
    """One attention head: SDDMM -> scores kept as fp32 -> row softmax in double
    -> alpha rounded to fp16 -> SpMM with alpha as the sparse values.
    Returns (scores_f32, alpha_f16, C, S)."""
    s64, _ = sddmm(rowptr, col, val, X, Y, nthreads=nthreads, want_scale=False)
    s32 = s64.astype(np.float32)
    alpha = edge_softmax(rowptr, s32.astype(np.float64), scale, nthreads=nthreads)
    a16 = alpha.astype(np.float16)
    C, S = spmm(rowptr, col, a16, B, nthreads=nthreads)
    return s32, a16, C, S


# ---------------------------------------------------------------------------
# Error measure used by the parity tests
# ---------------------------------------------------------------------------
def graded_error(got: np.ndarray, ref: np.ndarray, S: np.ndarray, terms) -> float:
    """max_e |got-ref| / max(|ref|, S/sqrt(d)).

    An output whose terms cancel to ~0 cannot be held to a pure relative
    error; S/sqrt(d) is the size a sum of d terms of total magnitude S would
    have with random signs, so ordinary outputs get a relative error and
    cancelled ones are measured against their natural scale.  ``terms`` is the
    number of summed terms per output (scalar, or broadcastable array)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    d = np.maximum(np.asarray(terms, dtype=np.float64), 1.0)
    den = np.maximum(np.abs(ref), S / np.sqrt(d))
    diff = np.abs(got - ref)
    with np.errstate(divide="ignore", invalid="ignore"):
        e = np.where(den > 0, diff / den, np.where(diff > 0, np.inf, 0.0))
    return float(e.max()) if e.size else 0.0
