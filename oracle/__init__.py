"""CPU oracle for Ozaki-scheme FP64 GEMM emulation on an INT8 matrix unit.

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the
benchmark's CPU-baseline leg.  The product (the HIP library and its Python
binding) never imports this package, and this package never imports the
product.  The arithmetic lives in ``ozaki_oracle.c`` (plain scalar C, int64 dot
products); this module only builds it with gcc and marshals numpy arrays.

Parity unpinned: none of the functions below (see tests/test_oracle_*.py for
the pins of each).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ozaki_oracle.c")
_LIB = os.path.join(_HERE, "liboz_oracle.so")
# A build of the same source made elsewhere (the sanitizer test points this at an instrumented build)
_LIB_OVERRIDE = os.environ.get("OZ_ORACLE_LIB")

_i64 = ctypes.c_int64
_int = ctypes.c_int
_vp = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (generic x86-64 + FMA for TwoProduct)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c99", "-O2", "-mfma", "-ffp-contract=off", "-fno-fast-math",
               "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        if _LIB_OVERRIDE:
            lib = ctypes.CDLL(_LIB_OVERRIDE)
        else:
            build()
            lib = ctypes.CDLL(_LIB)
        lib.oz_beta.argtypes = [_i64]
        lib.oz_beta.restype = _int
        lib.oz_r.argtypes = [_i64, _int]
        lib.oz_r.restype = _i64
        lib.oz_count_addends.argtypes = [_int, _i64]
        lib.oz_count_addends.restype = _i64
        lib.oz_row_exponents.argtypes = [_i64, _i64, _vp, _vp]
        lib.oz_row_exponents.restype = None
        lib.oz_col_exponents.argtypes = [_i64, _i64, _vp, _vp]
        lib.oz_col_exponents.restype = None
        lib.oz_split_rows.argtypes = [_i64, _i64, _vp, _vp, _int, _int, _int, _vp]
        lib.oz_split_rows.restype = None
        lib.oz_split_cols.argtypes = [_i64, _i64, _vp, _vp, _int, _int, _int, _vp]
        lib.oz_split_cols.restype = None
        lib.oz_group_chunk.argtypes = [_i64, _i64, _i64, _vp, _vp, _int, _int, _int, _vp]
        lib.oz_group_chunk.restype = _i64
        lib.oz_accumulate.argtypes = [_i64, _i64, _vp, _vp, _vp, _int, _int, _int, _vp]
        lib.oz_accumulate.restype = None
        lib.oz_dgemm.argtypes = [_i64, _i64, _i64, _vp, _vp, _int, _vp, _vp]
        lib.oz_dgemm.restype = _i64
        lib.oz_dot2_gemm.argtypes = [_i64, _i64, _i64, _vp, _vp, _vp, _vp]
        lib.oz_dot2_gemm.restype = None
        lib.oz_dgemm_variant.argtypes = [_i64, _i64, _i64, _vp, _vp, _int, _int, _int, _vp, _vp]
        lib.oz_dgemm_variant.restype = _i64
        lib.oz_exponents_floor.argtypes = [_i64, _i64, _vp, _int, _vp]
        lib.oz_exponents_floor.restype = None
        lib.oz_r_wide.argtypes = [_i64, _int]
        lib.oz_r_wide.restype = _i64
        lib.oz_axpby.argtypes = [_i64, _i64, ctypes.c_double, _vp, ctypes.c_double, _vp]
        lib.oz_axpby.restype = None
        lib.oz_split_per_slice.argtypes = [_i64, _i64, _vp, _int, _int, _int, _int, _vp, _vp]
        lib.oz_split_per_slice.restype = None
        lib.oz_dgemm_per_slice.argtypes = [_i64, _i64, _i64, _vp, _vp, _int, _vp, _vp]
        lib.oz_dgemm_per_slice.restype = _i64
        lib.oz_num_threads.argtypes = []
        lib.oz_num_threads.restype = _int
        _lib = lib
    return _lib


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _p(a: np.ndarray):
    return a.ctypes.data_as(_vp)


# ----------------------------------------------------------------------------
def params(n: int) -> Tuple[int, int]:
    """(beta, r) for inner dimension n  [the formulas for beta (Section 2) and r (Section 3.2)]."""
    lib = _load()
    beta = lib.oz_beta(int(n))
    return beta, int(lib.oz_r(int(n), beta))


def count_addends(k: int, r: int) -> int:
    """Number of FP64 additions per element, by walking Algorithm 6's loops."""
    return int(_load().oz_count_addends(int(k), int(r)))


def row_exponents(A: np.ndarray) -> np.ndarray:
    A = _c(A, np.float64)
    m, n = A.shape
    e = np.empty(m, dtype=np.int32)
    _load().oz_row_exponents(m, n, _p(A), _p(e))
    return e


def col_exponents(B: np.ndarray) -> np.ndarray:
    B = _c(B, np.float64)
    n, p = B.shape
    e = np.empty(p, dtype=np.int32)
    _load().oz_col_exponents(n, p, _p(B), _p(e))
    return e


_FORMS = {"int": 0, "sigma": 1, "bitmask": 2}


def exponents_floor(X: np.ndarray, by_col: bool) -> np.ndarray:
    """floor(log2 max |x|) per row (or per column) of X  [Algorithm 3, its scale mu'']; 0 for a zero vector."""
    X = _c(X, np.float64)
    rows, cols = X.shape
    e = np.empty(cols if by_col else rows, dtype=np.int32)
    _load().oz_exponents_floor(rows, cols, _p(X), 1 if by_col else 0, _p(e))
    return e


def r_wide(n: int, beta: int) -> int:
    """Products of round-to-nearest slices that fit one INT32 accumulator (option beyond the paper)."""
    return int(_load().oz_r_wide(int(n), int(beta)))


def split_rows(A: np.ndarray, k: int, beta: int, form: str = "int",
               eA: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """INT8 slices SA[k][m][n] of A and its row exponents  [Algorithm 8].

    form "int": exact integer-mantissa rounding; form "sigma": the
    floating-point recipe of Algorithm 8 ((a + sigma) - sigma)."""
    A = _c(A, np.float64)
    m, n = A.shape
    if eA is None:
        eA = exponents_floor(A, by_col=False) if form == "bitmask" else row_exponents(A)
    eA = _c(eA, np.int32)
    S = np.empty((k, m, n), dtype=np.int8)
    _load().oz_split_rows(m, n, _p(A), _p(eA), int(beta), int(k), _FORMS[form], _p(S))
    return S, eA


def split_cols(B: np.ndarray, k: int, beta: int, form: str = "int",
               eB: Optional[np.ndarray] = None) -> Tuple[np.ndarray, np.ndarray]:
    """INT8 slices SB[k][n][p] of B and its column exponents  [Algorithm 8 on B^T]."""
    B = _c(B, np.float64)
    n, p = B.shape
    if eB is None:
        eB = exponents_floor(B, by_col=True) if form == "bitmask" else col_exponents(B)
    eB = _c(eB, np.int32)
    S = np.empty((k, n, p), dtype=np.int8)
    _load().oz_split_cols(n, p, _p(B), _p(eB), int(beta), int(k), _FORMS[form], _p(S))
    return S, eB


def group_chunk(SA: np.ndarray, SB: np.ndarray, g: int, s0: int, s1: int) -> np.ndarray:
    """INT32 sum over s = s0..s1 of A''_s B''_{g-s}  [Algorithm 6 inner loop].

    Raises if any int64 dot-product sum does not fit INT32."""
    SA = _c(SA, np.int8)
    SB = _c(SB, np.int8)
    k, m, n = SA.shape
    k2, n2, p = SB.shape
    assert n == n2 and 1 <= s0 <= s1 <= g - 1 and g - s0 <= k2 and s1 <= k
    C = np.empty((m, p), dtype=np.int32)
    bad = _load().oz_group_chunk(m, n, p, _p(SA), _p(SB), int(g), int(s0), int(s1), _p(C))
    if bad:
        raise OverflowError(f"{bad} INT32 overflows in chunk g={g} s={s0}..{s1}")
    return C


def pair_product(SA: np.ndarray, SB: np.ndarray, s: int, t: int) -> np.ndarray:
    """A''_s B''_t as INT32  [Algorithm 4, the slice product]."""
    return group_chunk(SA, SB, s + t, s, s)


def accumulate(D: np.ndarray, C: np.ndarray, eA: np.ndarray, eB: np.ndarray,
               beta: int, g: int, first: bool) -> None:
    """In place D += 2^(2 - beta g) diag(2^eA) FP64(C) diag(2^eB)  [Algorithm 6, the accumulation step]."""
    assert D.dtype == np.float64 and D.flags.c_contiguous
    C = _c(C, np.int32)
    m, p = D.shape
    _load().oz_accumulate(m, p, _p(C), _p(_c(eA, np.int32)), _p(_c(eB, np.int32)),
                          int(beta), int(g), 1 if first else 0, _p(D))


def chunks(k: int, r: int):
    """The (g, s0, s1) chunks in the order Algorithm 6 visits them."""
    out = []
    for g in range(2, k + 2):
        q, s_open = 0, 1
        for s in range(1, g):
            q += 1
            if q == r or s == g - 1:
                out.append((g, s_open, s))
                q, s_open = 0, s + 1
    return out


def dgemm(A: np.ndarray, B: np.ndarray, k: int, return_addends: bool = False):
    """D = A B emulated with k INT8 slices  [Algorithm 8 + Algorithm 6]."""
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    m, n = A.shape
    n2, p = B.shape
    assert n == n2
    D = np.empty((m, p), dtype=np.float64)
    w = _i64(0)
    rc = _load().oz_dgemm(m, n, p, _p(A), _p(B), int(k), _p(D), ctypes.byref(w))
    if rc < 0:
        raise ValueError("arguments outside the method's domain")
    if rc > 0:
        raise OverflowError(f"{rc} INT32 overflows")
    return (D, int(w.value)) if return_addends else D


def dgemm_variant(A: np.ndarray, B: np.ndarray, k: int, split: str = "rn", accumulate: str = "grouped",
                  return_addends: bool = False):
    """The variants compared in Section 4: split "rn" (Algorithm 8) or "bitmask" (Algorithm 3);
    accumulate "grouped" (Algorithm 6, r of Section 3.2), "per_pair" (Algorithm 4) or "wide"
    (chunks of r_wide products, round-to-nearest slices only; beyond the paper).
    ("rn","grouped") = ozIMMU_H, ("bitmask","grouped") = ozIMMU_EF, ("bitmask","per_pair") = ozIMMU."""
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    m, n = A.shape
    n2, p = B.shape
    assert n == n2
    D = np.empty((m, p), dtype=np.float64)
    w = _i64(0)
    rc = _load().oz_dgemm_variant(m, n, p, _p(A), _p(B), int(k), {"rn": 0, "bitmask": 1}[split],
                                  {"grouped": 0, "per_pair": 1, "wide": 2}[accumulate], _p(D), ctypes.byref(w))
    if rc < 0:
        raise ValueError("arguments outside the method's domain")
    if rc > 0:
        raise OverflowError(f"{rc} INT32 overflows")
    return (D, int(w.value)) if return_addends else D


def split_per_slice(X: np.ndarray, k: int, beta: int, by_col: bool, form: str = "int"):
    """Algorithm 5: slices S[s-1] (shape of X) and per-slice scale exponents E[s-1][v], one vector per
    row of X (by_col False) or per column (by_col True).  Slice s has scale 2^(E[s-1][v] + 1 - beta)."""
    X = _c(X, np.float64)
    rows, cols = X.shape
    S = np.empty((k, rows, cols), dtype=np.int8)
    E = np.empty((k, cols if by_col else rows), dtype=np.int32)
    _load().oz_split_per_slice(rows, cols, _p(X), int(bool(by_col)), int(beta), int(k),
                               {"int": 0, "sigma": 1}[form], _p(S), _p(E))
    return S, E


def dgemm_per_slice(A: np.ndarray, B: np.ndarray, k: int, return_addends: bool = False):
    """ozIMMU_RN: Algorithm 5 slices, one FP64 addition per slice pair (Algorithm 4's order)."""
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    m, n = A.shape
    n2, p = B.shape
    assert n == n2
    D = np.empty((m, p), dtype=np.float64)
    w = _i64(0)
    rc = _load().oz_dgemm_per_slice(m, n, p, _p(A), _p(B), int(k), _p(D), ctypes.byref(w))
    if rc < 0:
        raise ValueError("arguments outside the method's domain")
    if rc > 0:
        raise OverflowError(f"{rc} INT32 overflows")
    return (D, int(w.value)) if return_addends else D


def dgemm_sub(A: np.ndarray, B: np.ndarray, k: int, I: Sequence[int], J: Sequence[int]) -> np.ndarray:
    """D[I][:, J] of the emulated product: needs only rows I of A and columns J
    of B, because scales are per row of A / per column of B and the inner
    dimension (hence beta and r) is unchanged."""
    return dgemm(np.ascontiguousarray(A[np.asarray(I)]), np.ascontiguousarray(B[:, np.asarray(J)]), k)


def gemm_ex(transA: bool, transB: bool, alpha: float, A: np.ndarray, B: np.ndarray, beta: float,
            C: np.ndarray, k: int) -> np.ndarray:
    """C <- alpha * op(A) op(B) + beta * C with the product emulated by k slices
    [steps (i)-(v) of Section 1]; op(X) = X or X^T.  Returns the new C."""
    opA = np.ascontiguousarray(A.T if transA else A, dtype=np.float64)
    opB = np.ascontiguousarray(B.T if transB else B, dtype=np.float64)
    D = dgemm(opA, opB, k)
    out = np.array(C, dtype=np.float64, order="C", copy=True)
    assert out.shape == D.shape
    _load().oz_axpby(D.shape[0], D.shape[1], float(alpha), _p(D), float(beta), _p(out))
    return out


def dot2_gemm(A: np.ndarray, B: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Compensated (Dot2) product, returned unevaluated as (hi, lo)."""
    A = _c(A, np.float64)
    B = _c(B, np.float64)
    m, n = A.shape
    n2, p = B.shape
    assert n == n2
    hi = np.empty((m, p), dtype=np.float64)
    lo = np.empty((m, p), dtype=np.float64)
    _load().oz_dot2_gemm(m, n, p, _p(A), _p(B), _p(hi), _p(lo))
    return hi, lo


def num_threads() -> int:
    return int(_load().oz_num_threads())
