"""CPU oracle for CSR SpMM (test infrastructure, not part of the product).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It wraps `spmm_oracle.c` (plain C, fp64, row by row; see that
file's header for what it follows in the paper and what pins it) via ctypes
and never touches the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmm_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_spmm.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the row split)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        p = ctypes.c_void_p
        i64 = ctypes.c_int64
        lib.oracle_spmm_csr.argtypes = [i64, i64, i64, p, p, p, p, p, p, ctypes.c_int]
        lib.oracle_spmm_csr.restype = ctypes.c_int
        lib.oracle_spmm_csr_rows.argtypes = [i64, i64, i64, p, p, p, p, p, i64, p, p]
        lib.oracle_spmm_csr_rows.restype = ctypes.c_int
        _lib = lib
    return _lib


def _check_inputs(M, K, N, rowptr, colidx, vals, B):
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int32)
    colidx = np.ascontiguousarray(colidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    B = np.ascontiguousarray(B, dtype=np.float32)
    if rowptr.shape != (M + 1,):
        raise ValueError("rowptr must have M+1 entries")
    nnz = int(rowptr[-1]) if M >= 0 else 0
    if rowptr[0] != 0 or np.any(np.diff(rowptr) < 0):
        raise ValueError("rowptr must start at 0 and be non-decreasing")
    if colidx.shape != (nnz,) or vals.shape != (nnz,):
        raise ValueError("colidx / vals must have rowptr[M] entries")
    if B.size != K * N:
        raise ValueError("B must be K x N")
    if nnz and (colidx.min() < 0 or colidx.max() >= K):
        raise ValueError("column index out of range")
    return rowptr, colidx, vals, B


def spmm_csr(M, K, N, rowptr, colidx, vals, B, nthreads: int = 1, bound: bool = True):
    """Return (C_ref, BND) as float64 [M, N] arrays (BND is None if bound=False)."""
    rowptr, colidx, vals, B = _check_inputs(M, K, N, rowptr, colidx, vals, B)
    C = np.empty((M, N), dtype=np.float64)
    BND = np.empty((M, N), dtype=np.float64) if bound else None
    rc = _load().oracle_spmm_csr(
        M, K, N, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, B.ctypes.data,
        C.ctypes.data, BND.ctypes.data if bound else None, int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return C, BND


def spmm_csr_rows(M, K, N, rowptr, colidx, vals, B, rows):
    """Rows `rows` of the result only: (C_ref, BND) float64 [len(rows), N]."""
    rowptr, colidx, vals, B = _check_inputs(M, K, N, rowptr, colidx, vals, B)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    C = np.empty((rows.size, N), dtype=np.float64)
    BND = np.empty((rows.size, N), dtype=np.float64)
    rc = _load().oracle_spmm_csr_rows(
        M, K, N, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, B.ctypes.data,
        rows.ctypes.data, rows.size, C.ctypes.data, BND.ctypes.data)
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return C, BND
