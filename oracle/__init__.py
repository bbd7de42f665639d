"""CPU oracle for CSR SPMM / SDDMM / FusedMM.  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around `csr_oracle.c` (plain C loops, FP64 accumulation,
OpenMP over rows; see that file's header for the definitions followed, the
readings taken and the parity pins).  Only `tests/`, the smoke check and the
benchmark's `cpu_baseline` leg may import this package; it imports nothing from
the HIP path.

Every function takes host numpy arrays and returns FP64 arrays
`(result, abs_sum)`, where `abs_sum` is the per-entry sum of |terms|.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csr_oracle.c")
_LIB = os.path.join(_HERE, "libcsr_oracle.so")

#: spec tolerance: |gpu - oracle| <= REL_TOL * sum|terms| for every output entry
REL_TOL = 1e-5


def build(force: bool = True) -> str:
    """Compile csr_oracle.c (gcc -O2, OpenMP, no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB):
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             _SRC, "-o", _LIB, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def _bind(path: str):
    """Load an oracle shared object and declare its signatures."""
    lib = ctypes.CDLL(path)
    i32, p = ctypes.c_int32, ctypes.c_void_p
    lib.oracle_spmm.argtypes = [i32, i32, i32, p, p, p, p, p, p, p, i32]
    lib.oracle_sddmm.argtypes = [i32, i32, i32, p, p, p, p, p, p, p, p, i32]
    lib.oracle_fusedmm.argtypes = [i32, i32, i32, i32, p, p, p, p, p, p, p, p, p, i32]
    lib.oracle_num_threads.restype = ctypes.c_int
    for f in (lib.oracle_spmm, lib.oracle_sddmm, lib.oracle_fusedmm):
        f.restype = None
    return lib


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        _lib = _bind(_LIB)
    return _lib


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _f32(a, shape=None) -> Optional[np.ndarray]:
    if a is None:
        return None
    a = np.ascontiguousarray(a, dtype=np.float32)
    if shape is not None and a.shape != shape:
        raise ValueError(f"operand has shape {a.shape}, expected {shape}")
    return a


def _check_csr(M: int, K: int, rowptr: np.ndarray, colidx: np.ndarray, vals: Optional[np.ndarray]):
    if rowptr.shape != (M + 1,) or rowptr[0] != 0:
        raise ValueError("rowptr must have M+1 entries and start at 0")
    if np.any(np.diff(rowptr) < 0):
        raise ValueError("rowptr must be non-decreasing")
    nnz = int(rowptr[M])
    if colidx.shape != (nnz,):
        raise ValueError("colidx must have rowptr[M] entries")
    if nnz and (colidx.min() < 0 or colidx.max() >= K):
        raise ValueError("colidx out of range")
    if vals is not None and vals.shape != (nnz,):
        raise ValueError("vals must have rowptr[M] entries")


def _rows(rows: Optional[Sequence[int]], M: int):
    if rows is None:
        return None, M
    r = _i32(rows)
    if r.size and (r.min() < 0 or r.max() >= M):
        raise ValueError("row list out of range")
    return r, int(r.size)


def spmm(M: int, K: int, N: int, rowptr, colidx, vals, B, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """O = S.B (eq. (2)); returns (O, abs) of shape (M or len(rows), N), FP64."""
    rowptr, colidx, vals = _i32(rowptr), _i32(colidx), _f32(vals)
    _check_csr(M, K, rowptr, colidx, vals)
    if vals is None:
        raise ValueError("SPMM needs vals")
    B = _f32(B, (K, N))
    r, R = _rows(rows, M)
    O = np.empty((R, N), dtype=np.float64)
    absO = np.empty((R, N), dtype=np.float64)
    _load().oracle_spmm(M, K, N, _p(rowptr), _p(colidx), _p(vals), _p(B), _p(O), _p(absO), _p(r), R)
    return O, absO


def sddmm(M: int, K: int, D: int, rowptr, colidx, vals, A, B, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """P = S (.) (A.B^T) on S's pattern (eq. (1), scaled by vals unless vals is None).

    Returns (P, abs) with nnz entries in CSR order; with `rows` given, entries of
    other rows are NaN."""
    rowptr, colidx, vals = _i32(rowptr), _i32(colidx), _f32(vals)
    _check_csr(M, K, rowptr, colidx, vals)
    A, B = _f32(A, (M, D)), _f32(B, (K, D))
    r, R = _rows(rows, M)
    nnz = int(rowptr[M])
    P = np.full(nnz, np.nan, dtype=np.float64)
    absP = np.full(nnz, np.nan, dtype=np.float64)
    _load().oracle_sddmm(M, K, D, _p(rowptr), _p(colidx), _p(vals), _p(A), _p(B), _p(P), _p(absP), _p(r), R)
    return P, absP


def fusedmm(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, rows=None):
    """O = (S (.) (A.B^T)).C (eq. (3)), scores kept in FP64; returns (O, abs), FP64."""
    rowptr, colidx, vals = _i32(rowptr), _i32(colidx), _f32(vals)
    _check_csr(M, K, rowptr, colidx, vals)
    A, B, C = _f32(A, (M, D)), _f32(B, (K, D)), _f32(C, (K, N))
    r, R = _rows(rows, M)
    O = np.empty((R, N), dtype=np.float64)
    absO = np.empty((R, N), dtype=np.float64)
    _load().oracle_fusedmm(M, K, D, N, _p(rowptr), _p(colidx), _p(vals), _p(A), _p(B), _p(C),
                           _p(O), _p(absO), _p(r), R)
    return O, absO


def fusedmm_unfused_fp32(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C):
    """SPMM(SDDMM(.)) with the sampled scores rounded to FP32 in between: what an
    unfused FP32 pipeline computes.  Used to bound how much that rounding matters."""
    P, _ = sddmm(M, K, D, rowptr, colidx, vals, A, B)
    return spmm(M, K, N, rowptr, colidx, P.astype(np.float32), C)


def within_tolerance(got, want: np.ndarray, abs_sum: np.ndarray, rel_tol: float = REL_TOL):
    """The parity rule: every entry satisfies |got - want| <= rel_tol * abs_sum.

    Returns (ok, worst) where worst = max |got - want| / abs_sum over entries with
    abs_sum > 0 (entries with abs_sum == 0 must match exactly)."""
    got = np.asarray(got, dtype=np.float64)
    err = np.abs(got - want)
    ok = bool(np.all(err <= rel_tol * abs_sum))
    nz = abs_sum > 0
    worst = float(np.max(err[nz] / abs_sum[nz])) if np.any(nz) else 0.0
    if np.any(~nz) and np.any(err[~nz] != 0):
        ok, worst = False, float("inf")
    if not np.all(np.isfinite(got)):
        ok, worst = False, float("inf")
    return ok, worst
