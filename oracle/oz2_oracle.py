"""Python face of the CPU oracle (oz2_oracle.c + constants.py).

TEST INFRASTRUCTURE ONLY: importable from tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg; never from the product path.  Nothing here touches
the GPU or the HIP library.

Each function wraps one stage of Algorithm 1 of the paper and only marshals
numpy arrays into the C routine that does the arithmetic; `gemm` chains the
stages in the order of Algorithm 1 and returns every intermediate, so that a
test can compare stage by stage.  FP32 inputs (SGEMM emulation) are widened to
FP64 before the integer stages; the widening is exact, so the scale shifts,
truncated integers and residues are those of the FP32 data.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

from . import constants as K

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oz2_oracle.c")
_LIB = os.path.join(_HERE, "liboz2_oracle.so")
_lib = None

BUILD_CMD = ["gcc", "-O2", "-fopenmp", "-ffp-contract=off", "-Wall", "-shared",
             "-fPIC", _SRC, "-o", _LIB, "-lm"]


def build(force: bool = False) -> str:
    """Compile oz2_oracle.c (always when force, else only if not built yet)."""
    global _lib
    if force or not os.path.exists(_LIB):
        subprocess.check_call(BUILD_CMD)
        _lib = None
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _i64(x) -> C.c_int64:
    return C.c_int64(int(x))


def num_threads() -> int:
    """Threads the C routines will use (OpenMP default)."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        return int(env.split(",")[0])
    return len(os.sched_getaffinity(0))


def _strides(X: np.ndarray, axis: int):
    """axis=0: one vector per row of X; axis=1: one vector per column."""
    assert X.ndim == 2 and X.dtype == np.float64 and X.flags.c_contiguous
    rows, cols = X.shape
    if axis == 0:
        return rows, cols, cols, 1
    return cols, rows, 1, cols


def shifts(X: np.ndarray, axis: int, Pfast: float):
    """Algorithm 1 line 1 (fast mode).  Returns (t, e, T) per vector."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    nv, ln, sv, sh = _strides(X, axis)
    t = np.zeros(nv, np.int32)
    e = np.zeros(nv, np.int32)
    T = np.zeros(nv, np.float64)
    _load().oz2o_shifts(_p(X), _i64(nv), _i64(ln), _i64(sv), _i64(sh),
                        C.c_double(Pfast), _p(t), _p(e), _p(T))
    return t, e, T


def residues(X: np.ndarray, axis: int, t: np.ndarray, p: Sequence[int]) -> np.ndarray:
    """Algorithm 1 lines 2-5.  Returns int8 [N][nv][len] (vector-major)."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    nv, ln, sv, sh = _strides(X, axis)
    t = np.ascontiguousarray(t, dtype=np.int32)
    pa = np.asarray(p, dtype=np.int32)
    out = np.empty((len(pa), nv, ln), np.int8)
    _load().oz2o_residues(_p(X), _i64(nv), _i64(ln), _i64(sv), _i64(sh),
                          _p(t), _p(pa), C.c_int(len(pa)), _p(out))
    return out


def int8_gemm_rows(Ares: np.ndarray, Bres: np.ndarray, rows: np.ndarray) -> np.ndarray:
    """Algorithm 1 line 6 for the listed rows.  Returns int32 [N][len(rows)][n]."""
    Ares = np.ascontiguousarray(Ares, dtype=np.int8)
    Bres = np.ascontiguousarray(Bres, dtype=np.int8)
    N, m, k = Ares.shape
    N2, n, k2 = Bres.shape
    assert N == N2 and k == k2
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    assert rows.size == 0 or (rows.min() >= 0 and rows.max() < m)
    out = np.empty((N, rows.size, n), np.int32)
    _load().oz2o_int8_gemm_rows(_p(Ares), _p(Bres), C.c_int(N), _i64(m), _i64(n),
                                _i64(k), _p(rows), _i64(rows.size), _p(out))
    return out


MAX_K = 1 << 17           # Section 4.3: longest contraction with exact INT32 accumulation


def int8_gemm_rows_blocked(Ares, Bres, rows, kblock: int = MAX_K) -> np.ndarray:
    """Block matrix multiplication for k > 2^17 (Section 4.3).  Returns int64 [N][len(rows)][n]."""
    Ares = np.ascontiguousarray(Ares, dtype=np.int8)
    Bres = np.ascontiguousarray(Bres, dtype=np.int8)
    N, m, k = Ares.shape
    _, n, _ = Bres.shape
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    out = np.empty((N, rows.size, n), np.int64)
    _load().oz2o_int8_gemm_rows_blocked(_p(Ares), _p(Bres), C.c_int(N), _i64(m), _i64(n), _i64(k),
                                        _i64(kblock), _p(rows), _i64(rows.size), _p(out))
    return out


def mod_reduce64(prod: np.ndarray, p: Sequence[int]) -> np.ndarray:
    prod = np.ascontiguousarray(prod, dtype=np.int64)
    N = prod.shape[0]
    pa = np.asarray(p, dtype=np.int32)
    U = np.empty(prod.shape, np.uint8)
    _load().oz2o_mod_reduce64(_p(prod), C.c_int(N), _i64(prod.size // N), _p(pa), _p(U))
    return U


def int8_gemm_entries(Ares, Bres, ii, jj) -> np.ndarray:
    """Algorithm 1 line 6 for scattered entries.  Returns int32 [N][count]."""
    Ares = np.ascontiguousarray(Ares, dtype=np.int8)
    Bres = np.ascontiguousarray(Bres, dtype=np.int8)
    N, m, k = Ares.shape
    _, n, _ = Bres.shape
    ii = np.ascontiguousarray(ii, dtype=np.int64)
    jj = np.ascontiguousarray(jj, dtype=np.int64)
    assert ii.shape == jj.shape
    out = np.empty((N, ii.size), np.int32)
    _load().oz2o_int8_gemm_entries(_p(Ares), _p(Bres), C.c_int(N), _i64(m), _i64(n),
                                   _i64(k), _p(ii), _p(jj), _i64(ii.size), _p(out))
    return out


def mod_reduce(prod: np.ndarray, p: Sequence[int]) -> np.ndarray:
    """Algorithm 1 line 7.  prod is int32 [N][...]; returns uint8 of same shape."""
    prod = np.ascontiguousarray(prod, dtype=np.int32)
    N = prod.shape[0]
    count = prod.size // N
    pa = np.asarray(p, dtype=np.int32)
    U = np.empty(prod.shape, np.uint8)
    _load().oz2o_mod_reduce(_p(prod), C.c_int(N), _i64(count), _p(pa), _p(U))
    return U


def crt_fold(U: np.ndarray, c: K.Constants) -> np.ndarray:
    """Algorithm 1 lines 8-11.  U is uint8 [N][...]; returns C'' (float64)."""
    U = np.ascontiguousarray(U, dtype=np.uint8)
    N = U.shape[0]
    count = U.size // N
    s1 = np.asarray(c.s1, np.float64)
    s2 = np.asarray(c.s2, np.float64)
    out = np.empty(U.shape[1:], np.float64)
    _load().oz2o_crt_fold(_p(U), C.c_int(N), _i64(count), _p(s1), _p(s2),
                          C.c_double(c.P1), C.c_double(c.P2), C.c_double(c.Pinv),
                          _p(out))
    return out


def unscale_rows(Cpp, tA_rows, tB, alpha=1.0, beta=0.0, Cin=None) -> np.ndarray:
    """Algorithm 1 line 12 + alpha/beta for [nrows][n] blocks."""
    Cpp = np.ascontiguousarray(Cpp, np.float64)
    nrows, n = Cpp.shape
    tA_rows = np.ascontiguousarray(tA_rows, np.int32)
    tB = np.ascontiguousarray(tB, np.int32)
    out = np.empty_like(Cpp)
    cin = None
    if beta != 0.0:
        cin = np.ascontiguousarray(Cin, np.float64)
        assert cin.shape == Cpp.shape
    _load().oz2o_unscale_rows(_p(Cpp), _p(tA_rows), _p(tB), _i64(nrows), _i64(n),
                              C.c_double(alpha), C.c_double(beta),
                              _p(cin) if cin is not None else None, _p(out))
    return out


def unscale_entries(Cpp, tsum, alpha=1.0, beta=0.0, Cin=None) -> np.ndarray:
    Cpp = np.ascontiguousarray(Cpp, np.float64).ravel()
    tsum = np.ascontiguousarray(tsum, np.int32).ravel()
    out = np.empty_like(Cpp)
    cin = None
    if beta != 0.0:
        cin = np.ascontiguousarray(Cin, np.float64).ravel()
    _load().oz2o_unscale_entries(_p(Cpp), _p(tsum), _i64(Cpp.size),
                                 C.c_double(alpha), C.c_double(beta),
                                 _p(cin) if cin is not None else None, _p(out))
    return out


def round_to_f32(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, np.float64)
    out = np.empty(x.shape, np.float32)
    _load().oz2o_round_to_f32(_p(x), _i64(x.size), _p(out))
    return out


def dd_rows(A: np.ndarray, B: np.ndarray, rows: np.ndarray):
    """Rows of A@B in double-double, and of |A|@|B|: (hi, lo, absprod)."""
    A = np.ascontiguousarray(A, np.float64)
    B = np.ascontiguousarray(B, np.float64)
    m, k = A.shape
    k2, n = B.shape
    assert k == k2
    rows = np.ascontiguousarray(rows, np.int64)
    hi = np.empty((rows.size, n), np.float64)
    lo = np.empty_like(hi)
    ab = np.empty_like(hi)
    _load().oz2o_dd_rows(_p(A), _i64(k), _p(B), _i64(n), _i64(n), _i64(k),
                         _p(rows), _i64(rows.size), _p(hi), _p(lo), _p(ab))
    return hi, lo, ab


def accu_prescale(X: np.ndarray, axis: int):
    """Accurate mode: (e, 7-bit matrix ceil(|x| 2^(5-e)) as int8 [nv][len])."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    nv, ln, sv, sh = _strides(X, axis)
    e = np.zeros(nv, np.int32)
    bar = np.empty((nv, ln), np.int8)
    _load().oz2o_accu_prescale(_p(X), _i64(nv), _i64(ln), _i64(sv), _i64(sh), _p(e), _p(bar))
    return e, bar


def accu_shift_from_max(e, cmax, Paccu: float, is_zero=None) -> np.ndarray:
    """t = (5 - e) + floor(P'_accu - 0.51 log2 max(c, 1)) per vector (0 for zero vectors)."""
    e = np.ascontiguousarray(e, np.int32)
    cmax = np.ascontiguousarray(cmax, np.int64)
    z = np.zeros(e.size, np.uint8) if is_zero is None else np.ascontiguousarray(is_zero, np.uint8)
    t = np.zeros(e.size, np.int32)
    _load().oz2o_accu_shifts(_p(e), _p(cmax), _p(z), _i64(e.size), C.c_double(Paccu), _p(t))
    return t


def accu_shifts(A64: np.ndarray, B64: np.ndarray, Paccu: float, kblock: int = MAX_K) -> Dict:
    """Accurate-mode scale vectors of Section 4.2: Cbar = Abar Bbar, then the shifts from its
    row and column maxima.  The product is a library matmul in FP64, which is exact here
    (entries are integers below 2^29).

    k > kblock (the longest contraction one INT32 product holds, Section 4.3): Cbar is the sum of
    the products Cbar_r over K ranges of kblock ("block matrix multiplication", last sentence of
    Section 4.3).  The bound chain of Section 4.2 needs an upper bound of max_j sum_h |a_ih||b_hj|
    only, and  max_j sum_r (Cbar_r)_ij <= sum_r max_j (Cbar_r)_ij,  so the row maximum of Cbar is
    replaced by the sum over the ranges of the row maxima of Cbar_r (columns alike): no matrix
    larger than one INT32 product is ever reduced.  For k <= kblock this is the paper's formula."""
    eA, Abar = accu_prescale(A64, 0)
    eB, Bbar = accu_prescale(B64, 1)
    m, k = A64.shape
    n = B64.shape[1]
    rmax = np.zeros(m, np.int64)
    cmax = np.zeros(n, np.int64)
    for k0 in range(0, k, kblock):
        Cbar = np.matmul(Abar[:, k0:k0 + kblock].astype(np.float64), Bbar[:, k0:k0 + kblock].astype(np.float64).T)
        if Cbar.size:
            rmax += Cbar.max(axis=1).astype(np.int64)
            cmax += Cbar.max(axis=0).astype(np.int64)
    zA = np.ascontiguousarray(~A64.any(axis=1), dtype=np.uint8)
    zB = np.ascontiguousarray(~B64.any(axis=0), dtype=np.uint8)
    tA = accu_shift_from_max(eA, rmax, Paccu, zA)
    tB = accu_shift_from_max(eB, cmax, Paccu, zB)
    return dict(tA=tA, tB=tB, eA=eA, eB=eB, Abar=Abar, Bbar=Bbar, rmax=rmax, cmax=cmax)


def prepare(A: np.ndarray, B: np.ndarray, num_moduli: int, is_double: bool = True,
            accurate: bool = False, kblock: int = MAX_K) -> Dict:
    """Algorithm 1 lines 1-5 on the whole of A and B (fast or accurate scale vectors)."""
    c = K.constants(num_moduli, is_double)
    A64 = np.ascontiguousarray(A, dtype=np.float64)
    B64 = np.ascontiguousarray(B, dtype=np.float64)
    if accurate:
        out = accu_shifts(A64, B64, c.Paccu, kblock)
        tA, tB = out["tA"], out["tB"]
    else:
        tA, eA, TA = shifts(A64, 0, c.Pfast)
        tB, eB, TB = shifts(B64, 1, c.Pfast)
        out = dict(tA=tA, tB=tB, eA=eA, eB=eB, TA=TA, TB=TB)
    out["consts"] = c
    out["Ares"] = residues(A64, 0, tA, c.p)
    out["Bres"] = residues(B64, 1, tB, c.p)
    return out


def finish_rows(prep: Dict, rows: np.ndarray, alpha=1.0, beta=0.0,
                Cin_rows: Optional[np.ndarray] = None) -> Dict:
    """Algorithm 1 lines 6-12 for the listed rows of C."""
    c = prep["consts"]
    rows = np.ascontiguousarray(rows, np.int64)
    if prep["Ares"].shape[2] > MAX_K:
        prod = int8_gemm_rows_blocked(prep["Ares"], prep["Bres"], rows)
        U = mod_reduce64(prod, c.p)
    else:
        prod = int8_gemm_rows(prep["Ares"], prep["Bres"], rows)
        U = mod_reduce(prod, c.p)
    Cpp = crt_fold(U, c)
    cin = None if Cin_rows is None else np.asarray(Cin_rows, np.float64)
    C64 = unscale_rows(Cpp, prep["tA"][rows], prep["tB"], float(alpha), float(beta), cin)
    out = C64 if c.is_double else round_to_f32(C64)
    return dict(prod=prod, U=U, Cpp=Cpp, C=out)


def finish_entries(prep: Dict, ii, jj, alpha=1.0, beta=0.0, Cin=None) -> Dict:
    """Algorithm 1 lines 6-12 for scattered entries (ii[c], jj[c]) of C."""
    c = prep["consts"]
    ii = np.asarray(ii, np.int64)
    jj = np.asarray(jj, np.int64)
    prod = int8_gemm_entries(prep["Ares"], prep["Bres"], ii, jj)
    U = mod_reduce(prod, c.p)
    Cpp = crt_fold(U, c)
    tsum = prep["tA"][ii] + prep["tB"][jj]
    cin = None if Cin is None else np.asarray(Cin, np.float64)
    C64 = unscale_entries(Cpp, tsum, float(alpha), float(beta), cin)
    out = C64 if c.is_double else round_to_f32(C64)
    return dict(prod=prod, U=U, Cpp=Cpp, C=out)


def gemm(A: np.ndarray, B: np.ndarray, num_moduli: int, alpha=1.0, beta=0.0,
         Cin: Optional[np.ndarray] = None, is_double: bool = True, accurate: bool = False) -> Dict:
    """The whole of Algorithm 1; returns every stage."""
    prep = prepare(A, B, num_moduli, is_double, accurate)
    rows = np.arange(np.asarray(A).shape[0], dtype=np.int64)
    fin = finish_rows(prep, rows, alpha, beta, Cin)
    prep.update(fin)
    return prep
