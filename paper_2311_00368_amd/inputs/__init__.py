"""Seeded synthetic inputs (CSR patterns and dense operands) for tests and benchmarks.

This module is infrastructure shared by the GPU path's tests, the CPU oracle's
tests and the benchmark; it contains no arithmetic of SPMM / SDDMM / FusedMM and
imports neither the HIP binding nor the oracle.  All arrays are host numpy
arrays: ``int32`` indices, ``float32`` values, dense matrices row-major
(paper, section "Matrix Storage Layout").

The paper's own workloads are randomized matrices at 70-90 % sparsity whose
files are not available (section "Sparse Matrix Collection"); `workload()`
builds the five synthetic stand-ins used throughout this repository.
"""
from __future__ import annotations

import ctypes
import math
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libcsrgen.so")

# stream ids: one independent random stream per array
STREAM_PATTERN, STREAM_VALS, STREAM_A, STREAM_B, STREAM_C, STREAM_ROWLEN = 0, 1, 2, 3, 4, 5


def build(force: bool = True) -> str:
    """Compile gen.c into libcsrgen.so next to it (gcc, OpenMP)."""
    if force or not os.path.exists(_LIB):
        subprocess.run(
            ["gcc", "-O2", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-shared", "-fPIC",
             _SRC, "-o", _LIB, "-lm"],
            check=True,
        )
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        u64, i32, f32, f64 = ctypes.c_uint64, ctypes.c_int32, ctypes.c_float, ctypes.c_double
        p = ctypes.c_void_p
        lib.gen_raw_u64.argtypes = [u64, u64, u64, u64, p]
        lib.gen_uniform_f32.argtypes = [u64, u64, u64, f32, f32, p]
        lib.gen_normal_f32.argtypes = [u64, u64, u64, p]
        lib.gen_bernoulli_csr.argtypes = [u64, u64, i32, i32, f64, p, p]
        lib.gen_lognormal_csr.argtypes = [u64, u64, u64, i32, i32, f64, f64, p, p]
        for f in (lib.gen_raw_u64, lib.gen_uniform_f32, lib.gen_normal_f32,
                  lib.gen_bernoulli_csr, lib.gen_lognormal_csr):
            f.restype = None
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def raw_u64(seed: int, stream: int, first: int, n: int) -> np.ndarray:
    out = np.empty(n, dtype=np.uint64)
    _load().gen_raw_u64(seed, stream, first, n, _ptr(out))
    return out


def uniform(seed: int, stream: int, shape, lo: float = -1.0, hi: float = 1.0) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().gen_uniform_f32(seed, stream, out.size, lo, hi, _ptr(out))
    return out


def normal(seed: int, stream: int, shape) -> np.ndarray:
    out = np.empty(shape, dtype=np.float32)
    _load().gen_normal_f32(seed, stream, out.size, _ptr(out))
    return out


def bernoulli_csr(seed: int, M: int, K: int, p: float, stream: int = STREAM_PATTERN):
    """Pattern with every entry kept independently with probability p; columns ascending."""
    rowptr = np.empty(M + 1, dtype=np.int32)
    _load().gen_bernoulli_csr(seed, stream, M, K, p, _ptr(rowptr), None)
    colidx = np.empty(int(rowptr[M]), dtype=np.int32)
    _load().gen_bernoulli_csr(seed, stream, M, K, p, _ptr(rowptr), _ptr(colidx))
    return rowptr, colidx


def lognormal_csr(seed: int, M: int, K: int, mean: float, sigma: float,
                  stream: int = STREAM_PATTERN, len_stream: int = STREAM_ROWLEN):
    """Pattern whose row lengths are log-normal with arithmetic mean `mean` (before
    clipping to [1, K]); columns uniform without replacement, ascending."""
    mu = math.log(mean) - 0.5 * sigma * sigma
    rowptr = np.empty(M + 1, dtype=np.int32)
    _load().gen_lognormal_csr(seed, stream, len_stream, M, K, mu, sigma, _ptr(rowptr), None)
    colidx = np.empty(int(rowptr[M]), dtype=np.int32)
    _load().gen_lognormal_csr(seed, stream, len_stream, M, K, mu, sigma, _ptr(rowptr), _ptr(colidx))
    return rowptr, colidx


# ---------------------------------------------------------------------------
# CSR <-> dense helpers (format only; paper Fig. 1 conventions: 0-based indices,
# values in row-major order, rowptr has M+1 entries with rowptr[M] = nnz)
# ---------------------------------------------------------------------------

def to_bf16(a: np.ndarray):
    """Round an FP32 array to bfloat16 (round to nearest, ties to even; NaN stays NaN).  Returns
    (bits, widened): the uint16 bit patterns, and the same values widened back to FP32 - what a consumer
    of the bfloat16 array sees.  Input preparation for the bfloat16 entry points, no arithmetic of the method."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    nan = np.isnan(a)
    bits = np.where(nan, (u >> np.uint32(16)) | np.uint32(0x40), rounded).astype(np.uint16)
    widened = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return bits, widened.reshape(a.shape)


def csr_from_dense(dense: np.ndarray):
    """Store the entries of `dense` that are != 0, row by row, columns ascending."""
    dense = np.asarray(dense)
    M, _ = dense.shape
    rows, cols = np.nonzero(dense)          # row-major order
    rowptr = np.zeros(M + 1, dtype=np.int32)
    np.add.at(rowptr, rows + 1, 1)
    rowptr = np.cumsum(rowptr, dtype=np.int64).astype(np.int32)
    return rowptr, cols.astype(np.int32), dense[rows, cols].astype(np.float32)


def csr_to_dense(M: int, K: int, rowptr, colidx, vals=None, dtype=np.float64) -> np.ndarray:
    """Scatter stored entries into an M x K array; duplicates are summed."""
    out = np.zeros((M, K), dtype=dtype)
    rows = np.repeat(np.arange(M), np.diff(rowptr))
    v = np.ones(len(colidx), dtype=dtype) if vals is None else np.asarray(vals, dtype=dtype)
    np.add.at(out, (rows, np.asarray(colidx)), v)
    return out


# ---------------------------------------------------------------------------
# The five synthetic workloads
# ---------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    M: int
    K: int
    rowptr: np.ndarray
    colidx: np.ndarray
    vals: np.ndarray
    ops: Dict[str, dict] = field(default_factory=dict)   # op name -> {"N"/"D": ..., operand arrays}
    recipe: str = ""

    @property
    def nnz(self) -> int:
        return int(self.rowptr[self.M])


WORKLOADS = ("tiny", "spmm4k", "sddmm4k", "fused8k_skew", "large16k")


def custom_workload(M: int, K: int, density: float, N: int, D: int, seed: int = 0) -> Workload:
    """Bernoulli pattern of the given density with U[-1,1] values and operands, all three
    operations (widths N and D): e.g. the paper's benchmark shapes, M/K/N/sparsity = 8k/8k/128/70 %
    is custom_workload(8192, 8192, 0.30, 128, 128)."""
    rp, ci = bernoulli_csr(seed, M, K, density)
    vals = uniform(seed, STREAM_VALS, len(ci))
    A = uniform(seed, STREAM_A, (M, D))
    B = uniform(seed, STREAM_B, (K, D))
    C = uniform(seed, STREAM_C, (K, N))
    ops = {"spmm": dict(N=N, B=C), "sddmm": dict(D=D, A=A, B=B), "fusedmm": dict(D=D, N=N, A=A, B=B, C=C)}
    return Workload(name=f"custom_{M}x{K}_p{density:g}_N{N}_D{D}", M=M, K=K, rowptr=rp, colidx=ci, vals=vals, ops=ops,
                    recipe=f"Bernoulli p={density:g}, vals U[-1,1], A,B x{D} and C x{N} U[-1,1]")


def workload(name: str, seed: int = 0, scale: float = 1.0) -> Workload:
    """Build one of the five named workloads.

    `scale` < 1 shrinks M and K (rounded to a multiple of 64) while keeping the
    density, value distributions and dense widths: used by CPU-only tests.
    """
    def sz(n):
        return max(64, int(round(n * scale / 64)) * 64)

    if name == "tiny":
        M = K = sz(512)
        rp, ci = bernoulli_csr(seed, M, K, 0.10)
        vals = uniform(seed, STREAM_VALS, len(ci))
        A = uniform(seed, STREAM_A, (M, 64))
        B = uniform(seed, STREAM_B, (K, 64))
        C = uniform(seed, STREAM_C, (K, 64))
        ops = {"spmm": dict(N=64, B=B), "sddmm": dict(D=64, A=A, B=B),
               "fusedmm": dict(D=64, N=64, A=A, B=B, C=C)}
        recipe = "Bernoulli p=0.10, vals U[-1,1], A,B,C x64 U[-1,1]"
    elif name == "spmm4k":
        M = K = sz(4096)
        rp, ci = bernoulli_csr(seed, M, K, 0.10)
        vals = uniform(seed, STREAM_VALS, len(ci))
        ops = {"spmm": dict(N=256, B=uniform(seed, STREAM_B, (K, 256)))}
        recipe = "Bernoulli p=0.10, vals U[-1,1], B x256 U[-1,1]"
    elif name == "sddmm4k":
        M = K = sz(4096)
        rp, ci = bernoulli_csr(seed, M, K, 0.30)
        vals = uniform(seed, STREAM_VALS, len(ci), 0.0, 1.0)
        ops = {"sddmm": dict(D=128, A=normal(seed, STREAM_A, (M, 128)),
                             B=normal(seed, STREAM_B, (K, 128)))}
        recipe = "Bernoulli p=0.30, vals U[0,1], A,B x128 N(0,1)"
    elif name == "fused8k_skew":
        M = K = sz(8192)
        rp, ci = lognormal_csr(seed, M, K, 819.0 * (K / 8192.0), 1.0)
        vals = uniform(seed, STREAM_VALS, len(ci))
        ops = {"fusedmm": dict(D=64, N=64, A=normal(seed, STREAM_A, (M, 64)),
                               B=normal(seed, STREAM_B, (K, 64)),
                               C=normal(seed, STREAM_C, (K, 64)))}
        recipe = "row nnz lognormal(mean 819*K/8192, sigma 1) clipped [1,K], vals U[-1,1], A,B,C x64 N(0,1)"
    elif name == "large16k":
        M = K = sz(16384)
        rp, ci = bernoulli_csr(seed, M, K, 0.20)
        vals = uniform(seed, STREAM_VALS, len(ci))
        A = uniform(seed, STREAM_A, (M, 64))
        Bd = uniform(seed, STREAM_B, (K, 64))          # FusedMM / SDDMM right operand, K x 64
        C = uniform(seed, STREAM_C, (K, 512))          # K x 512: SPMM's dense input and FusedMM's C
        ops = {"spmm": dict(N=512, B=C), "sddmm": dict(D=64, A=A, B=Bd),
               "fusedmm": dict(D=64, N=512, A=A, B=Bd, C=C)}
        recipe = "Bernoulli p=0.20, vals U[-1,1], A,B x64 and C x512 U[-1,1] (SPMM multiplies by the x512 array)"
    else:
        raise ValueError(f"unknown workload {name!r}; choose from {WORKLOADS}")
    return Workload(name=name, M=M, K=K, rowptr=rp, colidx=ci, vals=vals, ops=ops, recipe=recipe)
