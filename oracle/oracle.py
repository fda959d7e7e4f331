"""numpy front end of the C oracle (oracle/oracle.c) -- TEST INFRASTRUCTURE ONLY.

``sgemm_f64`` evaluates the definition of matmul from Sec. 5.2 of the paper,
C[i][j] = sum_p A[i][p] * B[p][j], with fp32 inputs widened to fp64 and an fp64 running
sum in ascending p (see the header of oracle.c).  This module only marshals numpy
arrays into that routine and derives the comparison metrics the parity tests use.
It never touches the GPU library.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        # Load what is built; compile only when nothing is there (a stale-looking timestamp must not start a
        # compiler from a process that may already hold the GPU: rebuilding is `python -m oracle.build`).
        path = _build.LIB if _build.LIB.exists() else _build.build()
        lib = ctypes.CDLL(str(path))
        i64, p = ctypes.c_int64, ctypes.c_void_p
        lib.oracle_sgemm_f64.argtypes = [i64, i64, i64, i64, p, i64, i64, p, i64, i64,
                                         p, i64, i64, p, p, i64, ctypes.c_int]
        lib.oracle_sgemm_f64.restype = ctypes.c_int
        lib.oracle_host_cores.restype = ctypes.c_int
        lib.oracle_saxpy_f64.argtypes = [i64, ctypes.c_float, p, p, p]
        lib.oracle_saxpy_f64.restype = ctypes.c_int
        _lib = lib
    return _lib


def host_cores() -> int:
    """Cores this process may run on (affinity mask if available, else online cores)."""
    try:
        return len(os.sched_getaffinity(0))
    except AttributeError:
        return int(_load().oracle_host_cores())


def _as3d(x: np.ndarray) -> np.ndarray:
    if x.dtype != np.float32:
        raise TypeError("oracle inputs must be float32")
    if x.ndim == 2:
        x = x[None]
    if x.ndim != 3:
        raise ValueError("expected a 2-D matrix or a 3-D batch")
    if x.strides[2] != 4 or x.strides[1] % 4 or x.strides[0] % 4:
        x = np.ascontiguousarray(x)
    return x


def sgemm_f64(a: np.ndarray, b: np.ndarray, rows=None, want_abs: bool = False, threads: int | None = None):
    """fp64 product of fp32 matrices a (m,k)·b (k,n), or of batches (B,m,k)·(B,k,n).

    rows: optional sequence of row indices; then only those rows of C are computed
    (output shape (..., len(rows), n)).  want_abs: also return S = |a|·|b| in fp64.
    Leading dimensions are taken from the arrays' strides, so row-padded views work.
    """
    squeeze = a.ndim == 2
    a3, b3 = _as3d(a), _as3d(b)
    batch, m, k = a3.shape
    if b3.shape[0] != batch or b3.shape[1] != k:
        raise ValueError(f"shape mismatch {a.shape} x {b.shape}")
    n = b3.shape[2]
    lda = a3.strides[1] // 4 if m > 1 else max(k, 1)
    ldb = b3.strides[1] // 4 if k > 1 else max(n, 1)
    sa = a3.strides[0] // 4 if batch > 1 else 0
    sb = b3.strides[0] // 4 if batch > 1 else 0
    lda, ldb = max(lda, k), max(ldb, n)
    if rows is None:
        rows_arr, nrows, rows_ptr = None, m, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
        nrows, rows_ptr = int(rows_arr.size), rows_arr.ctypes.data
    c = np.empty((batch, nrows, n), dtype=np.float64)
    s = np.empty_like(c) if want_abs else None
    if threads is None:
        threads = host_cores()
    rc = _load().oracle_sgemm_f64(batch, m, n, k, a3.ctypes.data, lda, sa, b3.ctypes.data, ldb, sb,
                                  c.ctypes.data, max(n, 1), nrows * max(n, 1),
                                  s.ctypes.data if want_abs else None, rows_ptr, nrows, int(threads))
    if rc != 0:
        raise RuntimeError(f"oracle_sgemm_f64 failed with code {rc}")
    if squeeze:
        c = c[0]
        s = s[0] if want_abs else None
    return (c, s) if want_abs else c


def saxpy_f64(alpha: float, x: np.ndarray, y: np.ndarray) -> np.ndarray:
    """fp64 value of alpha * x + y for fp32 vectors (axpy of Sec. 5.2 of the paper)."""
    if x.dtype != np.float32 or y.dtype != np.float32 or x.ndim != 1 or x.shape != y.shape:
        raise TypeError("x and y must be float32 vectors of equal length")
    x = np.ascontiguousarray(x)
    y = np.ascontiguousarray(y)
    z = np.empty(x.shape, dtype=np.float64)
    rc = _load().oracle_saxpy_f64(x.size, float(np.float32(alpha)), x.ctypes.data, y.ctypes.data, z.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_saxpy_f64 failed with code {rc}")
    return z


def parity_metrics(c_test: np.ndarray, c_ref: np.ndarray, s_abs: np.ndarray) -> dict:
    """Comparison of an fp32 result with the fp64 oracle result.

    max_ratio   = max |c_test - c_ref| / S over entries with S > 0 (per-element bound is 1e-5)
    zero_ok     = entries with S == 0 are exactly zero in c_test
    rel_fro     = ||c_test - c_ref||_F / ||c_ref||_F over all logical entries
    bit_exact   = c_test equals c_ref rounded to fp32, compared by value (+0 == -0)
    rel_fro_max_problem = for a batch (3-D arrays) the largest relative Frobenius error of a single problem,
                  reported next to the whole-batch figure, which is the one that is gated; equals rel_fro otherwise
    """
    ct = np.asarray(c_test, dtype=np.float64)
    diff = np.abs(ct - c_ref)
    pos = s_abs > 0
    max_ratio = float((diff[pos] / s_abs[pos]).max()) if pos.any() else 0.0
    zero_ok = bool(np.all(ct[~pos] == 0.0))
    den = float(np.sqrt(np.sum(c_ref * c_ref)))
    num = float(np.sqrt(np.sum(diff * diff)))
    rel_fro = num / den if den > 0 else (0.0 if num == 0 else float("inf"))
    bit_exact = bool(np.array_equal(np.asarray(c_test, dtype=np.float32), c_ref.astype(np.float32)))
    finite = bool(np.isfinite(ct).all())
    per_problem = rel_fro
    if c_ref.ndim == 3:
        axes = (1, 2)
        nums = np.sqrt(np.sum(diff * diff, axis=axes))
        dens = np.sqrt(np.sum(c_ref * c_ref, axis=axes))
        ratios = np.where(dens > 0, nums / np.where(dens > 0, dens, 1.0), np.where(nums == 0, 0.0, np.inf))
        per_problem = float(ratios.max()) if ratios.size else 0.0
    return {"max_ratio": max_ratio, "zero_ok": zero_ok, "rel_fro": rel_fro, "rel_fro_max_problem": per_problem,
            "bit_exact": bit_exact, "finite": finite}
