"""ctypes front end of the CPU oracle (``mttkrp_oracle.c``).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: only ``tests/``, the smoke check and
the benchmark's CPU-baseline leg may import this module.  It holds argument
marshalling and the comparison norm; the arithmetic is in the C file, which
follows the element-wise MTTKRP definition (paper Sec. II-B, Eq. (elem), with
lambda = 1).  Nothing here imports the HIP package.

Parity status: pinned.  The C routine by tests/test_oracle_pins.py; the two
error measures below (through which every parity assertion goes) by
hand-computed values and planted mistakes in tests/test_comparator_pins.py.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mttkrp_oracle.c")
_LIB = os.path.join(_HERE, "libmttkrp_oracle.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no GPU involved).  Returns the .so path."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC",
           "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC]
    subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64p = ctypes.POINTER(ctypes.c_int64)
        for name in ("oracle_mttkrp_f64", "oracle_mttkrp_f32",
                     "oracle_mttkrp_f64_native", "oracle_mttkrp_f32_native"):
            fn = getattr(lib, name)
            fn.restype = ctypes.c_int
            fn.argtypes = [ctypes.c_int, i64p, ctypes.c_void_p,
                           ctypes.POINTER(ctypes.c_void_p), ctypes.c_int,
                           ctypes.c_int, i64p, ctypes.c_int64, ctypes.c_void_p,
                           ctypes.c_void_p]
        lib.oracle_max_threads.restype = ctypes.c_int
        lib.oracle_long_double_mant_bits.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    """Number of OpenMP threads the oracle will use."""
    return int(_load().oracle_max_threads())


def long_double_mant_bits() -> int:
    return int(_load().oracle_long_double_mant_bits())


def mttkrp(X: np.ndarray, factors: Sequence[Optional[np.ndarray]], k: int,
           rows: Optional[Sequence[int]] = None, native_acc: bool = False,
           lam: Optional[np.ndarray] = None) -> np.ndarray:
    """Mode-``k`` (0-based) MTTKRP of a dense tensor, Eq. (elem); lambda = 1
    unless ``lam`` (R weights) is given.

    X        numpy array of shape (I_0, ..., I_{d-1}); its logical entry
             X[i_0, ..., i_{d-1}] is what the definition sums.  It is laid out
             first-index-fastest (Fortran order) before the C routine sees it.
    factors  list of d arrays, factors[m] of shape (I_m, R); factors[k] is
             never read and may be None.
    rows     optional list of output row indices; the result then has one row
             per requested index, in that order.
    native_acc  accumulate in the data type instead of long double.
    Returns  M of shape (I_k, R) (or (len(rows), R)), dtype of X.
    """
    lib = _load()
    if X.dtype == np.float64:
        ct, suffix = np.float64, "f64"
    elif X.dtype == np.float32:
        ct, suffix = np.float32, "f32"
    else:
        raise TypeError("oracle supports float64 and float32 only")
    d = X.ndim
    if len(factors) != d:
        raise ValueError("need one factor slot per mode")
    Xf = np.asfortranarray(X)
    dims = (ctypes.c_int64 * d)(*X.shape)
    R = None
    keep = []
    ptrs = (ctypes.c_void_p * d)()
    for m in range(d):
        if m == k:
            ptrs[m] = None
            continue
        A = factors[m]
        if A is None:
            raise ValueError("factor %d missing" % m)
        A = np.ascontiguousarray(A, dtype=ct)
        if A.ndim != 2 or A.shape[0] != X.shape[m]:
            raise ValueError("factor %d has shape %s" % (m, A.shape))
        if R is None:
            R = A.shape[1]
        elif A.shape[1] != R:
            raise ValueError("factors disagree on R")
        keep.append(A)
        ptrs[m] = A.ctypes.data
    if R is None:  # d == 1: the empty product; caller must say R via factors[k]
        if factors[k] is None:
            raise ValueError("cannot infer R")
        R = factors[k].shape[1]
    if rows is None:
        nrows = X.shape[k]
        rows_p = None
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows_arr.size
        rows_p = rows_arr.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))
    M = np.zeros((nrows, R), dtype=ct)
    lam_p = None
    if lam is not None:
        lam_arr = np.ascontiguousarray(lam, dtype=ct)
        if lam_arr.shape != (R,):
            raise ValueError("lam must hold R weights")
        lam_p = lam_arr.ctypes.data
    fn = getattr(lib, "oracle_mttkrp_" + suffix + ("_native" if native_acc else ""))
    rc = fn(d, dims, Xf.ctypes.data, ptrs, R, k, rows_p, nrows, lam_p, M.ctypes.data)
    if rc != 0:
        raise RuntimeError("oracle returned %d" % rc)
    return M


def normwise_rel_err(M_test: np.ndarray, M_ref: np.ndarray) -> float:
    """||M_test - M_ref||_F / ||M_ref||_F with sums in long double.

    If the reference norm is zero the test norm must be zero too (returns 0.0
    in that case and inf otherwise).
    """
    a = np.asarray(M_test, dtype=np.longdouble)
    b = np.asarray(M_ref, dtype=np.longdouble)
    if a.shape != b.shape:
        raise ValueError("shape mismatch %s vs %s" % (a.shape, b.shape))
    num = np.sqrt(np.sum((a - b) ** 2))
    den = np.sqrt(np.sum(b ** 2))
    if den == 0:
        return 0.0 if num == 0 else float("inf")
    return float(num / den)


def rowwise_rel_err(M_test: np.ndarray, M_ref: np.ndarray) -> float:
    """max over output rows n of ||M_test[n] - M_ref[n]||_2 / ||M_ref[n]||_2.

    The normwise error above can hide one wrong row of small norm under the
    norm of the whole matrix; row n of the result depends only on subtensor
    S_n^(k) (Sec. III), so every row is also held to the tolerance on its own.
    A row whose reference is all zero must be all zero (else inf).
    """
    a = np.asarray(M_test, dtype=np.longdouble)
    b = np.asarray(M_ref, dtype=np.longdouble)
    if a.shape != b.shape or a.ndim != 2:
        raise ValueError("need two matrices of one shape, got %s and %s" % (a.shape, b.shape))
    num = np.sqrt(np.sum((a - b) ** 2, axis=1))
    den = np.sqrt(np.sum(b ** 2, axis=1))
    worst = 0.0
    for n in range(a.shape[0]):
        if den[n] == 0:
            e = 0.0 if num[n] == 0 else float("inf")
        else:
            e = float(num[n] / den[n])
        if e != e:              # NaN: no later row may hide it
            return float("nan")
        worst = max(worst, e)
    return worst
