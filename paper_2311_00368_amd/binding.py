"""Python binding of the csrk C-ABI (include/csrk.h): argument marshalling only.

Every function takes torch CUDA tensors (torch is used for device memory and
streams, nothing else), checks dtype / shape / contiguity / device, and passes raw
device pointers plus the current HIP stream to the library.  All arithmetic runs in
the library's HIP kernels.  If `libcsrk.so` is missing or cannot be loaded the import
of a function from here raises: there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcsrk.so")

CSRK_OK = 0

_lib = None


class CsrkError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"csrk error {code}: {msg}")
        self.code = code


def load(build_if_missing: bool = True):
    """Load libcsrk.so (building it with hipcc first only if the file is absent)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise FileNotFoundError(f"{LIB_PATH} not built: run `python -m paper_2311_00368_amd.build`")
        from . import build as _build
        _build.build()
    lib = ctypes.CDLL(LIB_PATH)
    i, p = ctypes.c_int, ctypes.c_void_p
    lib.spmm_csr.argtypes = [i, i, i, p, p, p, p, p, p]
    lib.sddmm_csr.argtypes = [i, i, i, p, p, p, p, p, p, p]
    lib.fusedmm_csr.argtypes = [i, i, i, i, p, p, p, p, p, p, p, p]
    lib.spmm_csr_bf16.argtypes = [i, i, i, p, p, p, p, p, p]
    lib.sddmm_csr_bf16.argtypes = [i, i, i, p, p, p, p, p, p, p]
    lib.fusedmm_csr_bf16.argtypes = [i, i, i, i, p, p, p, p, p, p, p, p]
    lib.csrk_validate_csr.argtypes = [i, i, p, p, p, ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
    lib.csrk_plan_create.argtypes = [i, i, p, p, p, ctypes.POINTER(ctypes.c_void_p)]
    lib.csrk_plan_destroy.argtypes = [p]
    lib.csrk_plan_info.argtypes = [p, ctypes.POINTER(ctypes.c_longlong), ctypes.POINTER(ctypes.c_int),
                                   ctypes.POINTER(ctypes.c_int)]
    lib.spmm_csr_plan.argtypes = [p, i, p, p, p, p]
    lib.sddmm_csr_plan.argtypes = [p, i, p, p, p, p, p]
    lib.fusedmm_csr_plan.argtypes = [p, i, i, p, p, p, p, p, p]
    sz = ctypes.c_size_t
    lib.csrk_workspace_bytes.argtypes = [i, i, i, i, i, ctypes.POINTER(sz)]
    lib.spmm_csr_ws.argtypes = [i, i, i, p, p, p, p, p, p, sz, p]
    lib.sddmm_csr_ws.argtypes = [i, i, i, p, p, p, p, p, p, p, sz, p]
    lib.fusedmm_csr_ws.argtypes = [i, i, i, i, p, p, p, p, p, p, p, p, sz, p]
    lib.csrk_plan_reserve.argtypes = [p, i]
    lib.fusedmm_csr_static.argtypes = [i, i, i, i, p, p, p, p, p, p, p, p]
    lib.csrk_tile_phases.argtypes = [i, i, i, i, i, p, p, p, p, p, p, p, p, ctypes.POINTER(ctypes.c_double),
                                     ctypes.POINTER(ctypes.c_int)]
    lib.csrk_debug_row_rotation.argtypes = [p, p]
    lib.csrk_microbench.argtypes = [i, ctypes.POINTER(ctypes.c_double)]
    lib.csrk_release_workspace.argtypes = []
    lib.csrk_profile_enable.argtypes = [i]
    lib.csrk_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int), i,
                                         ctypes.POINTER(ctypes.c_int)]
    for f in (lib.spmm_csr, lib.sddmm_csr, lib.fusedmm_csr, lib.spmm_csr_bf16, lib.sddmm_csr_bf16, lib.fusedmm_csr_bf16,
              lib.csrk_validate_csr, lib.csrk_release_workspace, lib.csrk_plan_create, lib.csrk_plan_destroy,
              lib.csrk_plan_info, lib.spmm_csr_plan, lib.sddmm_csr_plan, lib.fusedmm_csr_plan,
              lib.csrk_profile_enable, lib.csrk_profile_collect, lib.csrk_workspace_bytes, lib.spmm_csr_ws,
              lib.sddmm_csr_ws, lib.fusedmm_csr_ws, lib.csrk_plan_reserve, lib.csrk_tile_phases,
              lib.csrk_debug_row_rotation, lib.fusedmm_csr_static, lib.csrk_microbench):
        f.restype = ctypes.c_int
    lib.csrk_last_error.restype = ctypes.c_char_p
    lib.csrk_version.restype = ctypes.c_char_p
    _lib = lib
    return lib


def _check(code: int):
    if code != CSRK_OK:
        raise CsrkError(code, load().csrk_last_error().decode())


def _dev_ptr(t: Optional[torch.Tensor], name: str, dtype, shape=None, device=None):
    if t is None:
        return None
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name} must be a CUDA tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name} must be {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if device is not None and t.device != device:
        raise ValueError(f"{name} is on {t.device}, expected {device}")
    return ctypes.c_void_p(t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def _csr_ptrs(M: int, rowptr, colidx, vals, need_vals: bool):
    dev = rowptr.device
    rp = _dev_ptr(rowptr, "rowptr", torch.int32, (M + 1,))
    nnz = colidx.numel()
    ci = _dev_ptr(colidx, "colidx", torch.int32, (nnz,), dev)
    if vals is None and need_vals:
        raise ValueError("vals is required")
    va = _dev_ptr(vals, "vals", torch.float32, (nnz,), dev)
    return dev, nnz, rp, ci, va


def csrk_version() -> str:
    return load().csrk_version().decode()


def csrk_last_error() -> str:
    return load().csrk_last_error().decode()


def spmm_csr(M: int, K: int, N: int, rowptr, colidx, vals, B, O=None) -> torch.Tensor:
    """O = S.B on the current stream; returns O (allocated M x N if not given)."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.spmm_csr(M, K, N, rp, ci, va, _dev_ptr(B, "B", torch.float32, (K, N), dev),
                            _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


def sddmm_csr(M: int, K: int, D: int, rowptr, colidx, vals, A, B, P=None) -> torch.Tensor:
    """P = S (.) (A.B^T) on S's pattern (vals=None: all-ones pattern); returns P (nnz floats).
    P may be `vals` itself for the in-place form."""
    lib = load()
    dev, nnz, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if P is None:
        P = torch.empty((nnz,), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.sddmm_csr(M, K, D, rp, ci, va, _dev_ptr(A, "A", torch.float32, (M, D), dev),
                             _dev_ptr(B, "B", torch.float32, (K, D), dev),
                             _dev_ptr(P, "P", torch.float32, (nnz,), dev), _stream(dev)))
    return P


def fusedmm_csr(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, O=None) -> torch.Tensor:
    """O = (S (.) (A.B^T)).C on the current stream; returns O (M x N)."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.fusedmm_csr(M, K, D, N, rp, ci, va, _dev_ptr(A, "A", torch.float32, (M, D), dev),
                               _dev_ptr(B, "B", torch.float32, (K, D), dev),
                               _dev_ptr(C, "C", torch.float32, (K, N), dev),
                               _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


CSRK_OP_SPMM, CSRK_OP_SDDMM, CSRK_OP_FUSEDMM = 1, 2, 3


FAMILY_NAMES = {0: "general, equal shares", 1: "general, whole rows", 2: "whole-row kernels", 3: "tiled narrow",
                4: "tiled wide", 5: "tiled SDDMM", 6: "schedule"}


def csrk_explain_choice(op: int, cus: int, M: int, K: int, N: int, D: int, nnz: int, longest_row: int,
                        planned: bool = False) -> int:
    """Which kernel family (CSRK_FAMILY_*, see FAMILY_NAMES) a call of this shape would take; host-only."""
    fam = ctypes.c_int(-1)
    _check(load().csrk_explain_choice(op, cus, M, K, N, D, ctypes.c_longlong(nnz), longest_row, 1 if planned else 0,
                                      ctypes.byref(fam)))
    return int(fam.value)


def csrk_workspace_bytes(op: int, M: int, K: int, N: int, D: int = 0) -> int:
    """Bytes of workspace that a *_csr_ws call of this operation (CSRK_OP_*) and shape may need on the current device."""
    out = ctypes.c_size_t(0)
    _check(load().csrk_workspace_bytes(op, M, K, N, D, ctypes.byref(out)))
    return int(out.value)


def _ws_ptr(workspace: torch.Tensor, dev):
    if not isinstance(workspace, torch.Tensor) or not workspace.is_cuda or workspace.device != dev:
        raise TypeError("workspace must be a CUDA tensor on the operands' device")
    if not workspace.is_contiguous():
        raise ValueError("workspace must be contiguous")
    return ctypes.c_void_p(workspace.data_ptr()), ctypes.c_size_t(workspace.numel() * workspace.element_size())


def spmm_csr_ws(M: int, K: int, N: int, rowptr, colidx, vals, B, workspace, O=None) -> torch.Tensor:
    """spmm_csr on the caller's workspace (a CUDA tensor of at least csrk_workspace_bytes(...) bytes)."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws, ws_bytes = _ws_ptr(workspace, dev)
    with torch.cuda.device(dev):
        _check(lib.spmm_csr_ws(M, K, N, rp, ci, va, _dev_ptr(B, "B", torch.float32, (K, N), dev),
                               _dev_ptr(O, "O", torch.float32, (M, N), dev), ws, ws_bytes, _stream(dev)))
    return O


def sddmm_csr_ws(M: int, K: int, D: int, rowptr, colidx, vals, A, B, workspace, P=None) -> torch.Tensor:
    """sddmm_csr on the caller's workspace."""
    lib = load()
    dev, nnz, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if P is None:
        P = torch.empty((nnz,), dtype=torch.float32, device=dev)
    ws, ws_bytes = _ws_ptr(workspace, dev)
    with torch.cuda.device(dev):
        _check(lib.sddmm_csr_ws(M, K, D, rp, ci, va, _dev_ptr(A, "A", torch.float32, (M, D), dev),
                                _dev_ptr(B, "B", torch.float32, (K, D), dev),
                                _dev_ptr(P, "P", torch.float32, (nnz,), dev), ws, ws_bytes, _stream(dev)))
    return P


def fusedmm_csr_ws(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, workspace, O=None) -> torch.Tensor:
    """fusedmm_csr on the caller's workspace."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    ws, ws_bytes = _ws_ptr(workspace, dev)
    with torch.cuda.device(dev):
        _check(lib.fusedmm_csr_ws(M, K, D, N, rp, ci, va, _dev_ptr(A, "A", torch.float32, (M, D), dev),
                                  _dev_ptr(B, "B", torch.float32, (K, D), dev),
                                  _dev_ptr(C, "C", torch.float32, (K, N), dev),
                                  _dev_ptr(O, "O", torch.float32, (M, N), dev), ws, ws_bytes, _stream(dev)))
    return O


def fusedmm_csr_static(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, O) -> torch.Tensor:
    """fusedmm_csr on the library's static scratch area: allocates nothing (O must be given)."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    with torch.cuda.device(dev):
        _check(lib.fusedmm_csr_static(M, K, D, N, rp, ci, va, _dev_ptr(A, "A", torch.float32, (M, D), dev),
                                      _dev_ptr(B, "B", torch.float32, (K, D), dev),
                                      _dev_ptr(C, "C", torch.float32, (K, N), dev),
                                      _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


def spmm_csr_bf16(M: int, K: int, N: int, rowptr, colidx, vals, B, O=None) -> torch.Tensor:
    """spmm_csr with B stored as bfloat16 (torch.bfloat16, K x N); O and vals are FP32."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.spmm_csr_bf16(M, K, N, rp, ci, va, _dev_ptr(B, "B", torch.bfloat16, (K, N), dev),
                                 _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


def sddmm_csr_bf16(M: int, K: int, D: int, rowptr, colidx, vals, A, B, P=None) -> torch.Tensor:
    """sddmm_csr with A (M x D) and B (K x D) stored as bfloat16; P and vals are FP32."""
    lib = load()
    dev, nnz, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if P is None:
        P = torch.empty((nnz,), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.sddmm_csr_bf16(M, K, D, rp, ci, va, _dev_ptr(A, "A", torch.bfloat16, (M, D), dev),
                                  _dev_ptr(B, "B", torch.bfloat16, (K, D), dev),
                                  _dev_ptr(P, "P", torch.float32, (nnz,), dev), _stream(dev)))
    return P


def fusedmm_csr_bf16(M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, O=None) -> torch.Tensor:
    """fusedmm_csr with A, B (x D) and C (K x N) stored as bfloat16; O and vals are FP32."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.fusedmm_csr_bf16(M, K, D, N, rp, ci, va, _dev_ptr(A, "A", torch.bfloat16, (M, D), dev),
                                    _dev_ptr(B, "B", torch.bfloat16, (K, D), dev),
                                    _dev_ptr(C, "C", torch.bfloat16, (K, N), dev),
                                    _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


class Plan:
    """A csrk_plan and the tensors it refers to (kept alive here; they must not be modified while the plan is
    in use).  Made by `csrk_plan_create`; destroyed with `csrk_plan_destroy` or when collected."""

    def __init__(self, handle, M, K, rowptr, colidx):
        self.handle, self.M, self.K, self.rowptr, self.colidx = handle, M, K, rowptr, colidx

    @property
    def device(self):
        return self.rowptr.device

    @property
    def nnz(self) -> int:
        return self.colidx.numel()

    def __del__(self):
        try:
            csrk_plan_destroy(self)
        except Exception:
            pass


def csrk_plan_create(M: int, K: int, rowptr, colidx) -> Plan:
    """Analyse the pattern once (synchronises the current stream); returns a Plan for the *_csr_plan calls."""
    lib = load()
    dev, _, rp, ci, _ = _csr_ptrs(M, rowptr, colidx, None, False)
    handle = ctypes.c_void_p(None)
    with torch.cuda.device(dev):
        _check(lib.csrk_plan_create(M, K, rp, ci, _stream(dev), ctypes.byref(handle)))
    return Plan(handle, M, K, rowptr, colidx)


def csrk_plan_destroy(plan: Plan) -> None:
    if plan.handle is not None and plan.handle.value:
        handle, plan.handle = plan.handle, None
        with torch.cuda.device(plan.device):
            _check(load().csrk_plan_destroy(handle))


PHASE_NAMES = ("barrier ending a tile", "tile copy to LDS", "barrier behind the copy", "tile loads issued",
               "accumulate stage", "next entries' loads issued", "score stage", "unused")


def csrk_tile_phases(op: int, M: int, K: int, D: int, N: int, rowptr, colidx, vals, A, B, C, O=None):
    """Mean cycles per wavefront and phase of the measuring build of the 512-column tiled SPMM / FusedMM kernel
    (see include/csrk.h).  Returns (cycles: list of 8 floats, tiles per wavefront, O)."""
    lib = load()
    dev, _, rp, ci, va = _csr_ptrs(M, rowptr, colidx, vals, False)
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    cycles = (ctypes.c_double * 8)()
    tiles = ctypes.c_int(0)
    with torch.cuda.device(dev):
        _check(lib.csrk_tile_phases(op, M, K, D, N, rp, ci, va,
                                    _dev_ptr(A, "A", torch.float32, (M, D), dev) if A is not None else None,
                                    _dev_ptr(B, "B", torch.float32, (K, D), dev) if B is not None else None,
                                    _dev_ptr(C, "C", torch.float32, (K, N), dev),
                                    _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev), cycles, ctypes.byref(tiles)))
    return list(cycles), int(tiles.value), O


def csrk_debug_row_rotation() -> torch.Tensor:
    """16 x 64 table: which lane's operand the rotated multiply-add hands to each lane (see include/csrk.h)."""
    out = torch.empty((16, 64), dtype=torch.float32, device="cuda")
    _check(load().csrk_debug_row_rotation(ctypes.c_void_p(out.data_ptr()), _stream(out.device)))
    return out


CSRK_BENCH_HBM_COPY, CSRK_BENCH_FMA_F32, CSRK_BENCH_LDS_READ = 1, 2, 3


def csrk_microbench(kind: int) -> float:
    """One of the library's machine-rate micro-benchmarks on the current device (see include/csrk.h): GB/s of a
    device copy, TFLOP/s of plain FP32 multiply-adds, or TB/s of 128-bit LDS reads."""
    out = ctypes.c_double(0.0)
    code = load().csrk_microbench(kind, ctypes.byref(out))
    if code != CSRK_OK:
        raise CsrkError(code, "csrk_microbench failed")
    return float(out.value)


def csrk_plan_reserve(plan: Plan, max_N: int) -> None:
    """Give the plan a workspace of its own for outputs of up to max_N columns (allocates; see include/csrk.h)."""
    with torch.cuda.device(plan.device):
        _check(load().csrk_plan_reserve(plan.handle, max_N))


def csrk_plan_info(plan: Plan):
    """(stored entries, columns strictly ascending in every row, rows even in length) as found at creation."""
    nnz, srt, even = ctypes.c_longlong(0), ctypes.c_int(0), ctypes.c_int(0)
    _check(load().csrk_plan_info(plan.handle, ctypes.byref(nnz), ctypes.byref(srt), ctypes.byref(even)))
    return nnz.value, bool(srt.value), bool(even.value)


def spmm_csr_plan(plan: Plan, N: int, vals, B, O=None) -> torch.Tensor:
    """spmm_csr on the plan's pattern."""
    lib, dev, M, K = load(), plan.device, plan.M, plan.K
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.spmm_csr_plan(plan.handle, N, _dev_ptr(vals, "vals", torch.float32, (plan.nnz,), dev),
                                 _dev_ptr(B, "B", torch.float32, (K, N), dev),
                                 _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


def sddmm_csr_plan(plan: Plan, D: int, vals, A, B, P=None) -> torch.Tensor:
    """sddmm_csr on the plan's pattern."""
    lib, dev, M, K = load(), plan.device, plan.M, plan.K
    if P is None:
        P = torch.empty((plan.nnz,), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.sddmm_csr_plan(plan.handle, D, _dev_ptr(vals, "vals", torch.float32, (plan.nnz,), dev),
                                  _dev_ptr(A, "A", torch.float32, (M, D), dev),
                                  _dev_ptr(B, "B", torch.float32, (K, D), dev),
                                  _dev_ptr(P, "P", torch.float32, (plan.nnz,), dev), _stream(dev)))
    return P


def fusedmm_csr_plan(plan: Plan, D: int, N: int, vals, A, B, C, O=None) -> torch.Tensor:
    """fusedmm_csr on the plan's pattern."""
    lib, dev, M, K = load(), plan.device, plan.M, plan.K
    if O is None:
        O = torch.empty((M, N), dtype=torch.float32, device=dev)
    with torch.cuda.device(dev):
        _check(lib.fusedmm_csr_plan(plan.handle, D, N, _dev_ptr(vals, "vals", torch.float32, (plan.nnz,), dev),
                                    _dev_ptr(A, "A", torch.float32, (M, D), dev),
                                    _dev_ptr(B, "B", torch.float32, (K, D), dev),
                                    _dev_ptr(C, "C", torch.float32, (K, N), dev),
                                    _dev_ptr(O, "O", torch.float32, (M, N), dev), _stream(dev)))
    return O


def csrk_validate_csr(M: int, K: int, rowptr, colidx) -> Tuple[int, bool]:
    """Device-side structural check; returns (problem bit mask, columns strictly ascending)."""
    lib = load()
    dev = rowptr.device
    rp = _dev_ptr(rowptr, "rowptr", torch.int32, (M + 1,))
    ci = _dev_ptr(colidx, "colidx", torch.int32, None, dev)
    problems, is_sorted = ctypes.c_int(0), ctypes.c_int(0)
    with torch.cuda.device(dev):
        _check(lib.csrk_validate_csr(M, K, rp, ci, _stream(dev), ctypes.byref(problems), ctypes.byref(is_sorted)))
    return problems.value, bool(is_sorted.value)


def csrk_release_workspace() -> None:
    _check(load().csrk_release_workspace())


def csrk_profile_enable(max_records: int) -> None:
    _check(load().csrk_profile_enable(max_records))


def csrk_profile_collect(capacity: int = 4096):
    """Returns [(kind, milliseconds), ...] for the recorded main-kernel launches, in call order
    (kind: 1 SPMM, 2 SDDMM, 3 FusedMM)."""
    ms = (ctypes.c_float * capacity)()
    kinds = (ctypes.c_int * capacity)()
    n = ctypes.c_int(0)
    _check(load().csrk_profile_collect(ms, kinds, capacity, ctypes.byref(n)))
    return [(kinds[t], ms[t]) for t in range(n.value)]
