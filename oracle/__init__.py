"""TEST INFRASTRUCTURE: the fp64 CPU checker for ``Y = A.X`` and ``A^l.X``.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares no code with the GPU library
and imports nothing from it.

* :func:`spmm`, :func:`spmm_iter`, :func:`sddmm`, :func:`mttkrp` -- ctypes wrappers of ``spmm_oracle.c``
  (plain CSR loops in fp64 over the original, undecomposed operand).
* :mod:`oracle.arrow_checks` -- host-side checks of a decomposition
  (bit-exact reassembly, arrow shape, injective permutations) and a slow
  evaluation of ``sum_i P_i^T B_i P_i X`` used to validate exported levels.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError(f"{_LIB_PATH} is missing: build it with "
                               "`python -m paper_2307_05740_amd._build oracle`")
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        lib.oracle_spmm.restype = ctypes.c_int
        lib.oracle_spmm.argtypes = [i64, vp, vp, vp, vp, i64, i32, i64, vp, vp, vp]
        lib.oracle_spmm_iter.restype = ctypes.c_int
        lib.oracle_spmm_iter.argtypes = [i64, vp, vp, vp, vp, i32, i32, vp, vp]
        lib.oracle_sddmm.restype = ctypes.c_int
        lib.oracle_sddmm.argtypes = [i64, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.oracle_mttkrp.restype = ctypes.c_int
        lib.oracle_mttkrp.argtypes = [i64, i64, i64, i64, vp, vp, vp, vp, vp, vp, i32, vp, vp]
        lib.oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _csr(rowptr, colidx, vals):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    assert rowptr.ndim == 1 and rowptr.shape[0] >= 1
    assert colidx.shape[0] == vals.shape[0] == int(rowptr[-1])
    return rowptr, colidx, vals


def spmm(rowptr, colidx, vals, X, rows=None, c0: int = 0, kc: int | None = None):
    """fp64 ``A.X`` and the bound ``|A|.|X|``.

    ``rows``: optional int64 array selecting output rows (result row r is row
    ``rows[r]`` of the product); ``c0, kc``: optional column slice of X.
    Returns ``(Y, B)``, both float64 of shape (len(rows) or n, kc).
    """
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    n = rowptr.shape[0] - 1
    assert X.dtype == np.float32 and X.ndim == 2 and X.flags.c_contiguous and X.shape[0] == n
    k = X.shape[1]
    kc = k - c0 if kc is None else kc
    assert 0 <= c0 and kc >= 1 and c0 + kc <= k
    if rows is None:
        nrows, rows_ptr = n, None
    else:
        rows = np.ascontiguousarray(rows, dtype=np.int64)
        nrows, rows_ptr = rows.shape[0], rows.ctypes.data
    Y = np.empty((nrows, kc), dtype=np.float64)
    B = np.empty((nrows, kc), dtype=np.float64)
    rc = _load().oracle_spmm(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
                             X.ctypes.data + 4 * c0, k, kc, nrows, rows_ptr,
                             Y.ctypes.data, B.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_spmm failed ({rc})")
    return Y, B


def spmm_iter(rowptr, colidx, vals, X, l: int):
    """fp64 ``A^l.X`` (never rounded to fp32 between products) and ``|A|^l.|X|``."""
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    n = rowptr.shape[0] - 1
    assert X.dtype == np.float32 and X.ndim == 2 and X.flags.c_contiguous and X.shape[0] == n
    k = X.shape[1]
    Xl = np.empty((n, k), dtype=np.float64)
    El = np.empty((n, k), dtype=np.float64)
    rc = _load().oracle_spmm_iter(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
                                  X.ctypes.data, k, l, Xl.ctypes.data, El.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_spmm_iter failed ({rc})")
    return Xl, El


def sddmm(rowptr, colidx, vals, U, V):
    """fp64 ``S[p] = a_p * <U[i,:], V[j,:]>`` on the pattern of A (CSR order) and its bound
    ``|a_p| * <|U[i,:]|, |V[j,:]|>``.  Returns ``(S, B)``, float64 arrays of length nnz."""
    rowptr, colidx, vals = _csr(rowptr, colidx, vals)
    n = rowptr.shape[0] - 1
    for M in (U, V):
        assert M.dtype == np.float32 and M.ndim == 2 and M.flags.c_contiguous and M.shape[0] == n
    assert U.shape == V.shape
    nnz = int(rowptr[-1])
    S = np.empty(nnz, dtype=np.float64)
    B = np.empty(nnz, dtype=np.float64)
    rc = _load().oracle_sddmm(n, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data,
                              U.ctypes.data, V.ctypes.data, U.shape[1], S.ctypes.data, B.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_sddmm failed ({rc})")
    return S, B


def mttkrp(dims, ti, tj, tk, tv, B, C):
    """fp64 ``A(i, a) = sum_{j,k} T(i,j,k) B(j,a) C(k,a)`` over the coordinate list of T and its
    bound ``sum |T| |B| |C|``.  Returns ``(A, E)``, float64 arrays of shape (I, R)."""
    I, J, K = (int(d) for d in dims)
    ti = np.ascontiguousarray(ti, dtype=np.int32)
    tj = np.ascontiguousarray(tj, dtype=np.int32)
    tk = np.ascontiguousarray(tk, dtype=np.int32)
    tv = np.ascontiguousarray(tv, dtype=np.float32)
    assert ti.shape == tj.shape == tk.shape == tv.shape and ti.ndim == 1
    for M, rows in ((B, J), (C, K)):
        assert M.dtype == np.float32 and M.ndim == 2 and M.flags.c_contiguous and M.shape[0] == rows
    assert B.shape[1] == C.shape[1]
    R = B.shape[1]
    A = np.empty((I, R), dtype=np.float64)
    E = np.empty((I, R), dtype=np.float64)
    rc = _load().oracle_mttkrp(I, J, K, ti.shape[0], ti.ctypes.data, tj.ctypes.data, tk.ctypes.data,
                               tv.ctypes.data, B.ctypes.data, C.ctypes.data, R, A.ctypes.data, E.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"oracle_mttkrp failed ({rc})")
    return A, E


def num_threads() -> int:
    return int(_load().oracle_num_threads())
