"""CPU oracles for CSR SpMM, CSR SDDMM and MTTKRP / TTM on compressed sparse
fibers (test infrastructure, not part of the product).

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package.  It wraps `spmm_oracle.c`, `sddmm_oracle.c` and
`tensor_oracle.c` (plain C, fp64, row by row; see those files' headers for
what they follow in the paper and what pins them) via ctypes and never touches
the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRCS = [os.path.join(_HERE, f) for f in ("spmm_oracle.c", "sddmm_oracle.c", "tensor_oracle.c")]
_LIB = os.path.join(_HERE, "liboracle_spmm.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (plain -O2, OpenMP for the row split)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < max(os.path.getmtime(f) for f in _SRCS):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               *_SRCS, "-o", _LIB, "-lm"]
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
        lib.oracle_sddmm_csr.argtypes = [i64, i64, i64, p, p, p, p, p, p, p, ctypes.c_int]
        lib.oracle_sddmm_csr.restype = ctypes.c_int
        lib.oracle_mttkrp_csf.argtypes = [i64, i64, i64, i64, p, p, p, p, p, p, p, p, p, ctypes.c_int]
        lib.oracle_mttkrp_csf.restype = ctypes.c_int
        lib.oracle_ttm_csf.argtypes = [i64, i64, i64, p, p, p, p, p, p, ctypes.c_int]
        lib.oracle_ttm_csf.restype = ctypes.c_int
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


def sddmm_csr(M, K, J, rowptr, colidx, vals, X1, X2T, nthreads: int = 1, bound: bool = True):
    """out[p] = vals[p] * <X1[row(p), :], X2T[colidx[p], :]> for every stored
    entry p.  Returns (out_ref, BND) as float64 arrays of rowptr[M] entries."""
    rowptr, colidx, vals, X2T = _check_inputs(M, K, J, rowptr, colidx, vals, X2T)
    X1 = np.ascontiguousarray(X1, dtype=np.float32)
    if X1.size != M * J:
        raise ValueError("X1 must be M x J")
    nnz = colidx.size
    out = np.empty(nnz, dtype=np.float64)
    BND = np.empty(nnz, dtype=np.float64) if bound else None
    rc = _load().oracle_sddmm_csr(
        M, K, J, rowptr.ctypes.data, colidx.ctypes.data, vals.ctypes.data, X1.ctypes.data, X2T.ctypes.data,
        out.ctypes.data, BND.ctypes.data if bound else None, int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out, BND


def _check_csf(I, K, L, fptr, fidx, eptr, eidx, vals):
    fptr = np.ascontiguousarray(fptr, dtype=np.int32)
    fidx = np.ascontiguousarray(fidx, dtype=np.int32)
    eptr = np.ascontiguousarray(eptr, dtype=np.int32)
    eidx = np.ascontiguousarray(eidx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    if fptr.shape != (I + 1,) or fptr[0] != 0 or np.any(np.diff(fptr) < 0):
        raise ValueError("fptr must have I+1 non-decreasing entries starting at 0")
    F = int(fptr[-1])
    if fidx.shape != (F,) or eptr.shape != (F + 1,) or eptr[0] != 0 or np.any(np.diff(eptr) < 0):
        raise ValueError("fidx must have fptr[I] entries, eptr one more, non-decreasing from 0")
    E = int(eptr[-1])
    if eidx.shape != (E,) or vals.shape != (E,):
        raise ValueError("eidx / vals must have eptr[F] entries")
    if F and (fidx.min() < 0 or fidx.max() >= K):
        raise ValueError("second index out of range")
    if E and (eidx.min() < 0 or eidx.max() >= L):
        raise ValueError("third index out of range")
    return fptr, fidx, eptr, eidx, vals


def mttkrp_csf(I, K, L, J, fptr, fidx, eptr, eidx, vals, X1, X2, nthreads: int = 1, bound: bool = True):
    """Y[i,j] = sum over the stored (i,k,l) of A[i,k,l] * X1[k,j] * X2[l,j].
    Returns (Y_ref, BND) as float64 [I, J] arrays."""
    fptr, fidx, eptr, eidx, vals = _check_csf(I, K, L, fptr, fidx, eptr, eidx, vals)
    X1 = np.ascontiguousarray(X1, dtype=np.float32)
    X2 = np.ascontiguousarray(X2, dtype=np.float32)
    if X1.size != K * J or X2.size != L * J:
        raise ValueError("X1 must be K x J and X2 L x J")
    Y = np.empty((I, J), dtype=np.float64)
    BND = np.empty((I, J), dtype=np.float64) if bound else None
    rc = _load().oracle_mttkrp_csf(
        I, K, L, J, fptr.ctypes.data, fidx.ctypes.data, eptr.ctypes.data, eidx.ctypes.data, vals.ctypes.data,
        X1.ctypes.data, X2.ctypes.data, Y.ctypes.data, BND.ctypes.data if bound else None, int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return Y, BND


def ttm_csf(I, Jdim, K, L, fptr, fidx, eptr, eidx, vals, X1, nthreads: int = 1, bound: bool = True):
    """Yf[f,l] = sum over the stored entries (i,j,k) of fiber f of A[i,j,k] * X1[k,l]:
    the rows Y[i, fidx[f], :] of the result, one per stored fiber.
    Returns (Yf_ref, BND) as float64 [F, L] arrays."""
    fptr, fidx, eptr, eidx, vals = _check_csf(I, Jdim, K, fptr, fidx, eptr, eidx, vals)
    X1 = np.ascontiguousarray(X1, dtype=np.float32)
    if X1.size != K * L:
        raise ValueError("X1 must be K x L")
    F = fidx.size
    Y = np.empty((F, L), dtype=np.float64)
    BND = np.empty((F, L), dtype=np.float64) if bound else None
    rc = _load().oracle_ttm_csf(
        F, K, L, eptr.ctypes.data, eidx.ctypes.data, vals.ctypes.data, X1.ctypes.data,
        Y.ctypes.data, BND.ctypes.data if bound else None, int(nthreads))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return Y, BND
