"""Thin Python binding of the C-ABI HIP library (include/ozimmu.h).

Argument marshalling only: every function forwards device pointers of torch
tensors and the current HIP stream to the entry point of the same name.  There
is no CPU fallback: importing this module without the built library, or calling
it without a GPU, raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libozimmu.so")
MAX_SLICES = 20
SCRATCH_BYTES = 512

if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2409_13313_amd.build` (needs hipcc)")

_lib = ctypes.CDLL(LIB_PATH)
_i64, _int, _vp, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t

_lib.ozimmu_status_string.argtypes = [_int]
_lib.ozimmu_status_string.restype = ctypes.c_char_p
_lib.ozimmu_params.argtypes = [_i64, ctypes.POINTER(_int), ctypes.POINTER(_i64)]
_lib.ozimmu_params.restype = _int
_lib.ozimmu_num_chunks.argtypes = [_i64, _int]
_lib.ozimmu_num_chunks.restype = _i64
_lib.ozimmu_slices_bytes.argtypes = [_i64, _i64, _int]
_lib.ozimmu_slices_bytes.restype = _sz
_lib.ozimmu_workspace_bytes.argtypes = [_i64, _i64, _i64, _int]
_lib.ozimmu_workspace_bytes.restype = _sz
_lib.ozimmu_workspace_bytes_min.argtypes = [_i64, _i64, _i64, _int]
_lib.ozimmu_workspace_bytes_min.restype = _sz
_lib.ozimmu_dgemm.argtypes = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _vp, _sz, _vp]
_lib.ozimmu_dgemm.restype = _int
_lib.ozimmu_dgemm_profiled.argtypes = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _vp, _sz, _vp,
                                       ctypes.POINTER(_vp)]
_lib.ozimmu_dgemm_profiled.restype = _int
_lib.ozimmu_gemm_ex.argtypes = [_int, _int, _i64, _i64, _i64, ctypes.c_double, _vp, _i64, _vp, _i64, ctypes.c_double,
                                _vp, _i64, _int, _vp, _sz, _vp]
_lib.ozimmu_gemm_ex.restype = _int
_lib.ozimmu_workspace_bytes_ex.argtypes = [_i64, _i64, _i64, _int]
_lib.ozimmu_workspace_bytes_ex.restype = _sz
_lib.ozimmu_dgemm_variant.argtypes = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _int, _int, _vp, _sz, _vp]
_lib.ozimmu_dgemm_variant.restype = _int
_lib.ozimmu_r_wide.argtypes = [_i64]
_lib.ozimmu_r_wide.restype = _i64
_lib.ozimmu_split_A_variant.argtypes = [_i64, _i64, _vp, _i64, _int, _int, _vp, _vp, _vp]
_lib.ozimmu_split_A_variant.restype = _int
_lib.ozimmu_split_B_variant.argtypes = [_i64, _i64, _vp, _i64, _int, _int, _vp, _vp, _vp]
_lib.ozimmu_split_B_variant.restype = _int
_lib.ozimmu_split_A.argtypes = [_i64, _i64, _vp, _i64, _int, _vp, _vp, _vp]
_lib.ozimmu_split_A.restype = _int
_lib.ozimmu_split_B.argtypes = [_i64, _i64, _vp, _i64, _int, _vp, _vp, _vp]
_lib.ozimmu_split_B.restype = _int
_lib.ozimmu_gemm_group.argtypes = [_i64, _i64, _i64, _vp, _int, _vp, _int, _int, _int, _int, _vp, _i64, _vp, _vp]
_lib.ozimmu_gemm_group.restype = _int
_lib.ozimmu_accumulate.argtypes = [_i64, _i64, _vp, _i64, _vp, _vp, _int, _int, _int, _vp, _i64, _vp]
_lib.ozimmu_accumulate.restype = _int
_lib.ozimmu_gemm_group_accumulate.argtypes = [_i64, _i64, _i64, _vp, _int, _vp, _int, _int, _int, _int,
                                              _vp, _vp, _int, _vp, _i64, _vp, _vp]
_lib.ozimmu_gemm_group_accumulate.restype = _int
_lib.ozimmu_workspace_bytes_variant.argtypes = [_i64, _i64, _i64, _int, _int]
_lib.ozimmu_workspace_bytes_variant.restype = _sz
_lib.ozimmu_remainder_bytes.argtypes = [_i64, _i64, _int]
_lib.ozimmu_remainder_bytes.restype = _sz
_lib.ozimmu_split_A_per_slice.argtypes = [_i64, _i64, _vp, _i64, _int, _vp, _vp, _vp, _vp]
_lib.ozimmu_split_A_per_slice.restype = _int
_lib.ozimmu_split_B_per_slice.argtypes = [_i64, _i64, _vp, _i64, _int, _vp, _vp, _vp, _vp]
_lib.ozimmu_split_B_per_slice.restype = _int
_lib.ozimmu_init.argtypes = []
_lib.ozimmu_init.restype = _int
_lib.ozimmu_dgemm_static.argtypes = [_i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _int, _vp]
_lib.ozimmu_dgemm_static.restype = _int
_lib.ozimmu_export_slices.argtypes = [_i64, _i64, _int, _vp, _vp, _vp]
_lib.ozimmu_export_slices.restype = _int

EXPORTS = ["ozimmu_status_string", "ozimmu_params", "ozimmu_num_chunks", "ozimmu_slices_bytes",
           "ozimmu_workspace_bytes", "ozimmu_dgemm", "ozimmu_dgemm_profiled", "ozimmu_gemm_ex", "ozimmu_workspace_bytes_ex", "ozimmu_dgemm_variant",
           "ozimmu_r_wide", "ozimmu_split_A_variant", "ozimmu_split_B_variant", "ozimmu_split_A", "ozimmu_split_B", "ozimmu_gemm_group",
           "ozimmu_accumulate", "ozimmu_gemm_group_accumulate", "ozimmu_export_slices",
           "ozimmu_workspace_bytes_variant", "ozimmu_remainder_bytes", "ozimmu_split_A_per_slice",
           "ozimmu_split_B_per_slice", "ozimmu_init", "ozimmu_dgemm_static", "ozimmu_workspace_bytes_min"]


SPLIT_MODES = {"rn": 0, "bitmask": 1, "per_slice": 2}
ACCUMULATE_MODES = {"grouped": 0, "per_pair": 1, "wide": 2}
SCHEDULES = {"auto": 0, "one_launch": 0x100, "split_inner": 0x200, "chunk_parallel": 0x400, "queue": 0x800}


class OzimmuError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"ozimmu status {status}: {status_string(status)}")


def _check(status: int) -> None:
    if status != 0:
        raise OzimmuError(status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> torch.Tensor:
    if not t.is_cuda:
        raise ValueError("tensor must live on the GPU")
    if t.dtype != dtype:
        raise ValueError(f"expected {dtype}, got {t.dtype}")
    return t


def _ld(t: torch.Tensor) -> int:
    """Leading dimension of a 2-D row-major view (last stride must be 1)."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("expected a 2-D tensor with unit stride along rows")
    return t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0), 1)


def status_string(status: int) -> str:
    return _lib.ozimmu_status_string(status).decode()


def params(n: int) -> Tuple[int, int]:
    beta, r = _int(0), _i64(0)
    _check(_lib.ozimmu_params(n, ctypes.byref(beta), ctypes.byref(r)))
    return beta.value, r.value


def num_chunks(n: int, k: int) -> int:
    return int(_lib.ozimmu_num_chunks(n, k))


def slices_bytes(rows: int, n: int, k: int) -> int:
    return int(_lib.ozimmu_slices_bytes(rows, n, k))


def workspace_bytes(m: int, n: int, p: int, k: int) -> int:
    return int(_lib.ozimmu_workspace_bytes(m, n, p, k))


def workspace_bytes_min(m: int, n: int, p: int, k: int) -> int:
    return int(_lib.ozimmu_workspace_bytes_min(m, n, p, k))


def alloc_workspace(m: int, n: int, p: int, k, device="cuda", split: str = "rn") -> torch.Tensor:
    """Workspace for calls with k slices; k may be a sequence of slice counts the workspace is to serve
    (the requirement is not monotone in k, so the largest k alone would not do)."""
    ks = [k] if isinstance(k, int) else list(k)
    nbytes = max(int(_lib.ozimmu_workspace_bytes_variant(m, n, p, kk, SPLIT_MODES[split])) for kk in ks)
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def dgemm(A: torch.Tensor, B: torch.Tensor, k: int, D: Optional[torch.Tensor] = None,
          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """D = A B emulated with k INT8 slices on the matrix cores."""
    _dev(A, torch.float64), _dev(B, torch.float64)
    m, n = A.shape
    n2, p = B.shape
    if n != n2:
        raise ValueError("inner dimensions differ")
    if D is None:
        D = torch.empty((m, p), dtype=torch.float64, device=A.device)
    _dev(D, torch.float64)
    if workspace is None:
        workspace = alloc_workspace(m, n, p, k, A.device)
    _check(_lib.ozimmu_dgemm(m, n, p, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), D.data_ptr(), _ld(D), k,
                             workspace.data_ptr(), workspace.numel(), _stream()))
    return D


def dgemm_profiled(A: torch.Tensor, B: torch.Tensor, k: int, D: torch.Tensor, workspace: torch.Tensor,
                   events) -> torch.Tensor:
    """dgemm that records three torch.cuda.Event objects (start, after split,
    end) on the current stream; the events must have been recorded once before
    so that their HIP handles exist."""
    _dev(A, torch.float64), _dev(B, torch.float64), _dev(D, torch.float64)
    m, n = A.shape
    p = B.shape[1]
    handles = (_vp * 3)(*[_vp(ev.cuda_event) if ev is not None else _vp(None) for ev in events])
    _check(_lib.ozimmu_dgemm_profiled(m, n, p, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), D.data_ptr(), _ld(D), k,
                                      workspace.data_ptr(), workspace.numel(), _stream(), handles))
    return D


def r_wide(n: int) -> int:
    return int(_lib.ozimmu_r_wide(n))


def dgemm_variant(A: torch.Tensor, B: torch.Tensor, k: int, split: str = "rn", accumulate: str = "grouped",
                  D: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                  schedule: str = "auto") -> torch.Tensor:
    """D = A B in one of the variants of Section 4 (see ozimmu_dgemm_variant in the header); schedule
    "one_launch" / "split_inner" forces how the schedule is run (same bits either way)."""
    _dev(A, torch.float64), _dev(B, torch.float64)
    m, n = A.shape
    n2, p = B.shape
    if n != n2:
        raise ValueError("inner dimensions differ")
    if D is None:
        D = torch.empty((m, p), dtype=torch.float64, device=A.device)
    if workspace is None:
        workspace = alloc_workspace(m, n, p, k, A.device, split)
    _check(_lib.ozimmu_dgemm_variant(m, n, p, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), D.data_ptr(), _ld(D), k,
                                     SPLIT_MODES[split], ACCUMULATE_MODES[accumulate] | SCHEDULES[schedule],
                                     workspace.data_ptr(),
                                     workspace.numel(), _stream()))
    return D


def gemm_ex(transA: bool, transB: bool, alpha: float, A: torch.Tensor, B: torch.Tensor, beta: float,
            C: torch.Tensor, k: int, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """C <- alpha * op(A) op(B) + beta * C in place (product emulated with k slices)."""
    _dev(A, torch.float64), _dev(B, torch.float64), _dev(C, torch.float64)
    m, n = (A.shape[1], A.shape[0]) if transA else A.shape
    n2, p = (B.shape[1], B.shape[0]) if transB else B.shape
    if n != n2 or tuple(C.shape) != (m, p):
        raise ValueError("shapes do not match")
    if workspace is None:
        workspace = torch.empty(max(int(_lib.ozimmu_workspace_bytes_ex(m, n, p, k)), 256), dtype=torch.uint8,
                                device=A.device)
    _check(_lib.ozimmu_gemm_ex(1 if transA else 0, 1 if transB else 0, m, n, p, alpha, A.data_ptr(), _ld(A),
                               B.data_ptr(), _ld(B), beta, C.data_ptr(), _ld(C), k, workspace.data_ptr(),
                               workspace.numel(), _stream()))
    return C


def split_A(A: torch.Tensor, k: int, split: str = "rn") -> Tuple[torch.Tensor, torch.Tensor]:
    """(packed slice stack, int32 row exponents) of A; split "per_slice": exponents [k][m] (Algorithm 5)."""
    _dev(A, torch.float64)
    m, n = A.shape
    SA = torch.empty(max(slices_bytes(m, n, k), 256), dtype=torch.int8, device=A.device)
    if split == "per_slice":
        eA = torch.empty((k, m), dtype=torch.int32, device=A.device)
        rem = torch.empty(max(int(_lib.ozimmu_remainder_bytes(m, n, 0)), 256), dtype=torch.uint8, device=A.device)
        _check(_lib.ozimmu_split_A_per_slice(m, n, A.data_ptr(), _ld(A), k, SA.data_ptr(), eA.data_ptr(),
                                             rem.data_ptr(), _stream()))
        return SA, eA
    eA = torch.empty(m, dtype=torch.int32, device=A.device)
    if split == "rn":
        _check(_lib.ozimmu_split_A(m, n, A.data_ptr(), _ld(A), k, SA.data_ptr(), eA.data_ptr(), _stream()))
    else:
        _check(_lib.ozimmu_split_A_variant(m, n, A.data_ptr(), _ld(A), k, SPLIT_MODES[split], SA.data_ptr(),
                                           eA.data_ptr(), _stream()))
    return SA, eA


def split_B(B: torch.Tensor, k: int, split: str = "rn") -> Tuple[torch.Tensor, torch.Tensor]:
    """(packed slice stack, int32 column exponents) of B; split "per_slice": exponents [k][p] (Algorithm 5)."""
    _dev(B, torch.float64)
    n, p = B.shape
    SB = torch.empty(max(slices_bytes(p, n, k), 256), dtype=torch.int8, device=B.device)
    if split == "per_slice":
        eB = torch.empty((k, p), dtype=torch.int32, device=B.device)
        rem = torch.empty(max(int(_lib.ozimmu_remainder_bytes(p, n, 1)), 256), dtype=torch.uint8, device=B.device)
        _check(_lib.ozimmu_split_B_per_slice(n, p, B.data_ptr(), _ld(B), k, SB.data_ptr(), eB.data_ptr(),
                                             rem.data_ptr(), _stream()))
        return SB, eB
    eB = torch.empty(p, dtype=torch.int32, device=B.device)
    if split == "rn":
        _check(_lib.ozimmu_split_B(n, p, B.data_ptr(), _ld(B), k, SB.data_ptr(), eB.data_ptr(), _stream()))
    else:
        _check(_lib.ozimmu_split_B_variant(n, p, B.data_ptr(), _ld(B), k, SPLIT_MODES[split], SB.data_ptr(),
                                           eB.data_ptr(), _stream()))
    return SB, eB


def alloc_scratch(device="cuda") -> torch.Tensor:
    return torch.empty(SCRATCH_BYTES, dtype=torch.uint8, device=device)


def gemm_group(m: int, n: int, p: int, SA: torch.Tensor, kA: int, SB: torch.Tensor, kB: int,
               g: int, s0: int, s1: int, C: Optional[torch.Tensor] = None,
               scratch: Optional[torch.Tensor] = None) -> torch.Tensor:
    if C is None:
        C = torch.empty((m, p), dtype=torch.int32, device=SA.device)
    _dev(C, torch.int32)
    if scratch is None:
        scratch = alloc_scratch(SA.device)
    _check(_lib.ozimmu_gemm_group(m, n, p, SA.data_ptr(), kA, SB.data_ptr(), kB, g, s0, s1,
                                  C.data_ptr(), _ld(C), scratch.data_ptr(), _stream()))
    return C


def accumulate(C: torch.Tensor, eA: torch.Tensor, eB: torch.Tensor, beta: int, g: int, first: bool,
               D: torch.Tensor) -> torch.Tensor:
    _dev(C, torch.int32), _dev(D, torch.float64), _dev(eA, torch.int32), _dev(eB, torch.int32)
    m, p = D.shape
    _check(_lib.ozimmu_accumulate(m, p, C.data_ptr(), _ld(C), eA.data_ptr(), eB.data_ptr(), beta, g,
                                  1 if first else 0, D.data_ptr(), _ld(D), _stream()))
    return D


def gemm_group_accumulate(m: int, n: int, p: int, SA: torch.Tensor, kA: int, SB: torch.Tensor, kB: int,
                          g: int, s0: int, s1: int, eA: torch.Tensor, eB: torch.Tensor, first: bool,
                          D: torch.Tensor, scratch: Optional[torch.Tensor] = None) -> torch.Tensor:
    _dev(D, torch.float64)
    if scratch is None:
        scratch = alloc_scratch(SA.device)
    _check(_lib.ozimmu_gemm_group_accumulate(m, n, p, SA.data_ptr(), kA, SB.data_ptr(), kB, g, s0, s1,
                                             eA.data_ptr(), eB.data_ptr(), 1 if first else 0,
                                             D.data_ptr(), _ld(D), scratch.data_ptr(), _stream()))
    return D


def init() -> None:
    """One-time set-up of the current device (needed before the first library call inside a graph capture)."""
    _check(_lib.ozimmu_init())


STATIC_WORKSPACE_BYTES = 64 << 20


def dgemm_static(A: torch.Tensor, B: torch.Tensor, k: int, D: torch.Tensor) -> torch.Tensor:
    """dgemm on the library's static workspace: the call allocates nothing (D is the caller's)."""
    _dev(A, torch.float64), _dev(B, torch.float64), _dev(D, torch.float64)
    m, n = A.shape
    n2, p = B.shape
    if n != n2 or tuple(D.shape) != (m, p):
        raise ValueError("shapes do not match")
    _check(_lib.ozimmu_dgemm_static(m, n, p, A.data_ptr(), _ld(A), B.data_ptr(), _ld(B), D.data_ptr(), _ld(D), k,
                                    _stream()))
    return D


def export_slices(rows: int, n: int, k: int, packed: torch.Tensor) -> torch.Tensor:
    """Canonical int8 [k][rows][n] view of a packed stack (for B: [k][p][n])."""
    out = torch.empty((k, rows, n), dtype=torch.int8, device=packed.device)
    _check(_lib.ozimmu_export_slices(rows, n, k, packed.data_ptr(), out.data_ptr(), _stream()))
    return out
