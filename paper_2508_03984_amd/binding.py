"""ctypes binding of liboz2.so: same names as the C ABI (include/oz2.h),
argument marshalling only.  Device buffers are torch tensors; the stream is
torch's current stream unless given.  There is no fallback: if the library has
not been built, every call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "liboz2.so")
_lib = None

OZ2_STAGE_SHIFT_A, OZ2_STAGE_SHIFT_B, OZ2_STAGE_RES_A, OZ2_STAGE_RES_B, OZ2_STAGE_PROD, OZ2_STAGE_U = range(6)

EXPORTS = [
    "oz2_dgemm", "oz2_sgemm", "oz2_dgemm_accurate", "oz2_sgemm_accurate", "oz2_shift_table_accurate",
    "oz2_workspace_bytes", "oz2_set_workspace", "oz2_release",
    "oz2_constants", "oz2_shift_table", "oz2_stage_ptr", "oz2_int8_gemm", "oz2_set_profiling",
    "oz2_last_stage_times_ms", "oz2_status_string", "oz2_set_int32_products", "oz2_mfma_probe",
    "oz2_dgemm_op", "oz2_sgemm_op", "oz2_prepare_d", "oz2_prepare_s", "oz2_operand_free",
    "oz2_operand_bytes", "oz2_dgemm_prepared", "oz2_sgemm_prepared", "oz2_workspace_min_bytes",
    "oz2_set_workspace_limit", "oz2_last_panels", "oz2_last_gemm_launches", "oz2_ctx_last_gemm_launches", "oz2_plan_panels", "oz2_set_overlap",
    "oz2_set_small_conversion", "oz2_dgemm_colmajor", "oz2_sgemm_colmajor", "oz2_residue_rounds",
    "oz2_create", "oz2_destroy", "oz2_ctx_set_option", "oz2_ctx_dgemm", "oz2_ctx_sgemm",
    "oz2_ctx_dgemm_prepared", "oz2_ctx_sgemm_prepared", "oz2_ctx_workspace_bytes",
    "oz2_ctx_workspace_min_bytes", "oz2_ctx_set_workspace", "oz2_ctx_set_workspace_limit",
    "oz2_ctx_plan_panels", "oz2_ctx_last_panels", "oz2_ctx_release", "oz2_ctx_stage_ptr",
    "oz2_ctx_last_stage_times_ms", "oz2_dgemm_noalloc",
]

OZ2_OPT_INT32_PRODUCTS, OZ2_OPT_OVERLAP, OZ2_OPT_SMALL_CONVERSION, OZ2_OPT_PROFILING, OZ2_OPT_CUT_LAUNCHES = range(5)

OZ2_OP_N, OZ2_OP_T = 0, 1


class OZ2Error(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {oz2_status_string(status)} (status {status})")


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load liboz2.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    try:
        # torch ships its own HIP runtime under the same soname; importing it first makes the
        # loader bind liboz2.so to that one, so that streams and pointers are shared.
        import torch  # noqa: F401
    except ImportError:
        pass
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2508_03984_amd.build` "
            "(or __graft_entry__.build()); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    i64, dbl, flt, vp, ci = C.c_int64, C.c_double, C.c_float, C.c_void_p, C.c_int
    lib.oz2_dgemm.argtypes = [i64, i64, i64, dbl, vp, i64, vp, i64, dbl, vp, i64, ci, vp]
    lib.oz2_sgemm.argtypes = [i64, i64, i64, flt, vp, i64, vp, i64, flt, vp, i64, ci, vp]
    lib.oz2_dgemm_accurate.argtypes = lib.oz2_dgemm.argtypes
    lib.oz2_dgemm_noalloc.argtypes = lib.oz2_dgemm.argtypes
    lib.oz2_dgemm_noalloc.restype = ci
    lib.oz2_sgemm_accurate.argtypes = lib.oz2_sgemm.argtypes
    lib.oz2_shift_table_accurate.argtypes = [ci, vp, vp, vp, vp]
    lib.oz2_dgemm_op.argtypes = [ci, ci, ci] + lib.oz2_dgemm.argtypes
    lib.oz2_sgemm_op.argtypes = [ci, ci, ci] + lib.oz2_sgemm.argtypes
    lib.oz2_dgemm_colmajor.argtypes = lib.oz2_dgemm_op.argtypes
    lib.oz2_sgemm_colmajor.argtypes = lib.oz2_sgemm_op.argtypes
    lib.oz2_prepare_d.argtypes = [ci, ci, i64, i64, vp, i64, ci, vp, C.POINTER(vp)]
    lib.oz2_prepare_s.argtypes = lib.oz2_prepare_d.argtypes
    lib.oz2_operand_free.argtypes = [vp]
    lib.oz2_operand_free.restype = None
    lib.oz2_operand_bytes.argtypes = [vp]
    lib.oz2_operand_bytes.restype = C.c_size_t
    lib.oz2_dgemm_prepared.argtypes = [vp, vp, dbl, dbl, vp, i64, vp]
    lib.oz2_sgemm_prepared.argtypes = [vp, vp, flt, flt, vp, i64, vp]
    lib.oz2_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    lib.oz2_workspace_bytes.restype = C.c_size_t
    lib.oz2_workspace_min_bytes.argtypes = [i64, i64, i64, ci, ci]
    lib.oz2_workspace_min_bytes.restype = C.c_size_t
    lib.oz2_set_workspace_limit.argtypes = [C.c_size_t]
    lib.oz2_set_workspace_limit.restype = None
    lib.oz2_last_panels.argtypes = [C.POINTER(i64), C.POINTER(i64), C.POINTER(i64)]
    lib.oz2_plan_panels.argtypes = [i64, i64, i64, ci, C.c_size_t] + lib.oz2_last_panels.argtypes
    lib.oz2_set_workspace.argtypes = [vp, C.c_size_t]
    lib.oz2_release.argtypes = []
    lib.oz2_release.restype = None
    lib.oz2_constants.argtypes = [ci, ci, vp, vp, vp, vp, vp, vp]
    lib.oz2_shift_table.argtypes = [ci, vp, vp, vp]
    lib.oz2_stage_ptr.argtypes = [ci, C.POINTER(vp), C.POINTER(i64)]
    lib.oz2_int8_gemm.argtypes = [vp, vp, vp, ci, i64, i64, i64, vp]
    lib.oz2_mfma_probe.argtypes = [ci, C.c_double, C.POINTER(C.c_double), C.POINTER(ci), C.POINTER(ci)]
    lib.oz2_set_profiling.argtypes = [ci]
    lib.oz2_set_profiling.restype = None
    lib.oz2_set_int32_products.argtypes = [ci]
    lib.oz2_set_int32_products.restype = None
    lib.oz2_set_overlap.argtypes = [ci]
    lib.oz2_set_overlap.restype = None
    lib.oz2_set_small_conversion.argtypes = [ci]
    lib.oz2_set_small_conversion.restype = None
    lib.oz2_last_stage_times_ms.argtypes = [C.POINTER(flt)]
    lib.oz2_create.argtypes = [C.POINTER(vp)]
    lib.oz2_destroy.argtypes = [vp]
    lib.oz2_ctx_set_option.argtypes = [vp, ci, ci]
    lib.oz2_ctx_dgemm.argtypes = [vp, ci, ci, ci] + lib.oz2_dgemm.argtypes
    lib.oz2_ctx_sgemm.argtypes = [vp, ci, ci, ci] + lib.oz2_sgemm.argtypes
    lib.oz2_ctx_dgemm_prepared.argtypes = [vp] + lib.oz2_dgemm_prepared.argtypes
    lib.oz2_ctx_sgemm_prepared.argtypes = [vp] + lib.oz2_sgemm_prepared.argtypes
    lib.oz2_ctx_workspace_bytes.argtypes = [vp, i64, i64, i64, ci]
    lib.oz2_ctx_workspace_bytes.restype = C.c_size_t
    lib.oz2_ctx_workspace_min_bytes.argtypes = [vp, i64, i64, i64, ci]
    lib.oz2_ctx_workspace_min_bytes.restype = C.c_size_t
    lib.oz2_ctx_set_workspace.argtypes = [vp, vp, C.c_size_t]
    lib.oz2_ctx_set_workspace_limit.argtypes = [vp, C.c_size_t]
    lib.oz2_ctx_plan_panels.argtypes = [vp] + lib.oz2_plan_panels.argtypes
    lib.oz2_ctx_last_panels.argtypes = [vp] + lib.oz2_last_panels.argtypes
    lib.oz2_last_gemm_launches.argtypes = [C.POINTER(i64)]
    lib.oz2_ctx_last_gemm_launches.argtypes = [vp, C.POINTER(i64)]
    lib.oz2_ctx_release.argtypes = [vp]
    lib.oz2_ctx_stage_ptr.argtypes = [vp] + lib.oz2_stage_ptr.argtypes
    lib.oz2_ctx_last_stage_times_ms.argtypes = [vp, C.POINTER(flt)]
    for name in EXPORTS:
        if name.startswith("oz2_ctx_") or name in ("oz2_create", "oz2_destroy"):
            getattr(lib, name).restype = ci
    lib.oz2_ctx_workspace_bytes.restype = C.c_size_t
    lib.oz2_ctx_workspace_min_bytes.restype = C.c_size_t
    lib.oz2_residue_rounds.argtypes = [ci, ci]
    lib.oz2_residue_rounds.restype = ci
    lib.oz2_status_string.argtypes = [ci]
    lib.oz2_status_string.restype = C.c_char_p
    for name in ("oz2_dgemm", "oz2_sgemm", "oz2_dgemm_accurate", "oz2_sgemm_accurate",
                 "oz2_shift_table_accurate", "oz2_set_workspace", "oz2_constants", "oz2_shift_table",
                 "oz2_stage_ptr", "oz2_int8_gemm", "oz2_last_stage_times_ms", "oz2_mfma_probe",
                 "oz2_dgemm_op", "oz2_sgemm_op", "oz2_prepare_d", "oz2_prepare_s", "oz2_dgemm_prepared",
                 "oz2_sgemm_prepared", "oz2_last_panels", "oz2_plan_panels", "oz2_dgemm_colmajor",
                 "oz2_sgemm_colmajor"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _stream(stream) -> C.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return C.c_void_p(int(stream))


def _dev(t, dtype=None) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"tensor of dtype {dtype} expected, got {t.dtype}")
    return C.c_void_p(t.data_ptr())


def _check(status: int, where: str) -> None:
    if status != 0:
        raise OZ2Error(status, where)


def oz2_status_string(status: int) -> str:
    return load().oz2_status_string(int(status)).decode()


def oz2_dgemm(m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli, stream=None) -> None:
    import torch
    _check(load().oz2_dgemm(m, n, k, float(alpha), _dev(A, torch.float64), lda,
                            _dev(B, torch.float64), ldb, float(beta), _dev(C_, torch.float64), ldc,
                            int(num_moduli), _stream(stream)), "oz2_dgemm")


OZ2_NOALLOC_WORKSPACE_BYTES = 64 * 1024 * 1024


def oz2_dgemm_noalloc(m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli, stream=None) -> None:
    import torch
    _check(load().oz2_dgemm_noalloc(m, n, k, float(alpha), _dev(A, torch.float64), lda,
                                    _dev(B, torch.float64), ldb, float(beta), _dev(C_, torch.float64), ldc,
                                    int(num_moduli), _stream(stream)), "oz2_dgemm_noalloc")


def oz2_sgemm(m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli, stream=None) -> None:
    import torch
    _check(load().oz2_sgemm(m, n, k, float(alpha), _dev(A, torch.float32), lda,
                            _dev(B, torch.float32), ldb, float(beta), _dev(C_, torch.float32), ldc,
                            int(num_moduli), _stream(stream)), "oz2_sgemm")


def oz2_dgemm_accurate(m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli, stream=None) -> None:
    import torch
    _check(load().oz2_dgemm_accurate(m, n, k, float(alpha), _dev(A, torch.float64), lda,
                                     _dev(B, torch.float64), ldb, float(beta),
                                     _dev(C_, torch.float64), ldc, int(num_moduli), _stream(stream)),
           "oz2_dgemm_accurate")


def oz2_sgemm_accurate(m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli, stream=None) -> None:
    import torch
    _check(load().oz2_sgemm_accurate(m, n, k, float(alpha), _dev(A, torch.float32), lda,
                                     _dev(B, torch.float32), ldb, float(beta),
                                     _dev(C_, torch.float32), ldc, int(num_moduli), _stream(stream)),
           "oz2_sgemm_accurate")


def oz2_dgemm_op(opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                 stream=None) -> None:
    import torch
    _check(load().oz2_dgemm_op(int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                               _dev(A, torch.float64), lda, _dev(B, torch.float64), ldb, float(beta),
                               _dev(C_, torch.float64), ldc, int(num_moduli), _stream(stream)),
           "oz2_dgemm_op")


def oz2_sgemm_op(opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                 stream=None) -> None:
    import torch
    _check(load().oz2_sgemm_op(int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                               _dev(A, torch.float32), lda, _dev(B, torch.float32), ldb, float(beta),
                               _dev(C_, torch.float32), ldc, int(num_moduli), _stream(stream)),
           "oz2_sgemm_op")


def oz2_dgemm_colmajor(opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                       stream=None) -> None:
    import torch
    _check(load().oz2_dgemm_colmajor(int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                                     _dev(A, torch.float64), lda, _dev(B, torch.float64), ldb, float(beta),
                                     _dev(C_, torch.float64), ldc, int(num_moduli), _stream(stream)),
           "oz2_dgemm_colmajor")


def oz2_sgemm_colmajor(opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                       stream=None) -> None:
    import torch
    _check(load().oz2_sgemm_colmajor(int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                                     _dev(A, torch.float32), lda, _dev(B, torch.float32), ldb, float(beta),
                                     _dev(C_, torch.float32), ldc, int(num_moduli), _stream(stream)),
           "oz2_sgemm_colmajor")


class Operand:
    """Owner of an oz2_operand handle (oz2_prepare_d / oz2_prepare_s); freed with the object."""

    def __init__(self, handle: int, side: int, rows: int, k: int, is_double: bool):
        self.handle, self.side, self.rows, self.k, self.is_double = handle, side, rows, k, is_double

    @property
    def nbytes(self) -> int:
        return int(load().oz2_operand_bytes(C.c_void_p(self.handle)))

    def free(self) -> None:
        if self.handle:
            load().oz2_operand_free(C.c_void_p(self.handle))
            self.handle = 0

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def _prepare(fn_name, dtype, side, op, rows, k, X, ld, num_moduli, stream) -> Operand:
    out = C.c_void_p(0)
    _check(getattr(load(), fn_name)(int(side), int(op), rows, k, _dev(X, dtype), ld, int(num_moduli),
                                    _stream(stream), C.byref(out)), fn_name)
    return Operand(int(out.value), int(side), rows, k, fn_name.endswith("_d"))


def oz2_prepare_d(side, op, rows, k, X, ld, num_moduli, stream=None) -> Operand:
    import torch
    return _prepare("oz2_prepare_d", torch.float64, side, op, rows, k, X, ld, num_moduli, stream)


def oz2_prepare_s(side, op, rows, k, X, ld, num_moduli, stream=None) -> Operand:
    import torch
    return _prepare("oz2_prepare_s", torch.float32, side, op, rows, k, X, ld, num_moduli, stream)


def oz2_operand_free(operand: Operand) -> None:
    operand.free()


def oz2_operand_bytes(operand: Operand) -> int:
    return operand.nbytes


def oz2_dgemm_prepared(left: Operand, right: Operand, alpha, beta, C_, ldc, stream=None) -> None:
    import torch
    _check(load().oz2_dgemm_prepared(C.c_void_p(left.handle), C.c_void_p(right.handle), float(alpha),
                                     float(beta), _dev(C_, torch.float64), ldc, _stream(stream)),
           "oz2_dgemm_prepared")


def oz2_sgemm_prepared(left: Operand, right: Operand, alpha, beta, C_, ldc, stream=None) -> None:
    import torch
    _check(load().oz2_sgemm_prepared(C.c_void_p(left.handle), C.c_void_p(right.handle), float(alpha),
                                     float(beta), _dev(C_, torch.float32), ldc, _stream(stream)),
           "oz2_sgemm_prepared")


def oz2_workspace_min_bytes(m, n, k, num_moduli, is_double=True) -> int:
    return int(load().oz2_workspace_min_bytes(m, n, k, int(num_moduli), int(bool(is_double))))


def oz2_set_workspace_limit(nbytes: int) -> None:
    load().oz2_set_workspace_limit(int(nbytes))


def oz2_last_panels() -> Tuple[int, int, int]:
    pr, pc, cnt = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load().oz2_last_panels(C.byref(pr), C.byref(pc), C.byref(cnt)), "oz2_last_panels")
    return int(pr.value), int(pc.value), int(cnt.value)


def oz2_plan_panels(m, n, k, num_moduli, workspace_bytes) -> Tuple[int, int, int]:
    pr, pc, cnt = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load().oz2_plan_panels(m, n, k, int(num_moduli), int(workspace_bytes), C.byref(pr), C.byref(pc),
                                  C.byref(cnt)), "oz2_plan_panels")
    return int(pr.value), int(pc.value), int(cnt.value)


def oz2_shift_table_accurate(num_moduli: int) -> dict:
    import numpy as np
    pa = np.zeros(1, np.float32); f = np.zeros(1, np.int32); lv = np.zeros(1, np.int32)
    th = np.zeros(20, np.uint64)
    _check(load().oz2_shift_table_accurate(int(num_moduli), pa.ctypes.data, f.ctypes.data,
                                           lv.ctypes.data, th.ctypes.data), "oz2_shift_table_accurate")
    return dict(Paccu=float(pa[0]), f_max=int(f[0]), levels=int(lv[0]), theta=th[:int(lv[0])].copy())


def oz2_workspace_bytes(m, n, k, num_moduli, is_double=True) -> int:
    return int(load().oz2_workspace_bytes(m, n, k, int(num_moduli), int(bool(is_double))))


def oz2_set_workspace(buf) -> None:
    """buf: a device uint8 tensor the caller keeps alive, or None for library-owned."""
    if buf is None:
        _check(load().oz2_set_workspace(C.c_void_p(0), 0), "oz2_set_workspace")
    else:
        _check(load().oz2_set_workspace(_dev(buf), buf.numel() * buf.element_size()),
               "oz2_set_workspace")


def oz2_release() -> None:
    load().oz2_release()


def oz2_constants(num_moduli: int, is_double: bool = True) -> dict:
    import numpy as np
    n = int(num_moduli)
    p = np.zeros(20, np.int32); pv = np.zeros(20, np.uint32)
    s1 = np.zeros(20, np.float64); s2 = np.zeros(20, np.float64)
    P = np.zeros(3, np.float64); pf = np.zeros(1, np.float32)
    _check(load().oz2_constants(n, int(bool(is_double)), p.ctypes.data, pv.ctypes.data,
                                s1.ctypes.data, s2.ctypes.data, P.ctypes.data, pf.ctypes.data),
           "oz2_constants")
    return dict(p=p[:n], pinv_prime=pv[:n], s1=s1[:n], s2=s2[:n], P1=float(P[0]), P2=float(P[1]),
                Pinv=float(P[2]), Pfast=float(pf[0]))


def oz2_shift_table(num_moduli: int) -> dict:
    import numpy as np
    f = np.zeros(1, np.int32); lv = np.zeros(1, np.int32); th = np.zeros(20, np.uint64)
    _check(load().oz2_shift_table(int(num_moduli), f.ctypes.data, lv.ctypes.data, th.ctypes.data),
           "oz2_shift_table")
    return dict(f_max=int(f[0]), levels=int(lv[0]), theta=th[:int(lv[0])].copy())


def oz2_residue_rounds(num_moduli: int, accurate: bool = False) -> int:
    return int(load().oz2_residue_rounds(int(num_moduli), int(bool(accurate))))


def oz2_stage_ptr(stage: int) -> Tuple[int, Tuple[int, int, int, int]]:
    ptr = C.c_void_p(0)
    dims = (C.c_int64 * 4)()
    _check(load().oz2_stage_ptr(int(stage), C.byref(ptr), dims), "oz2_stage_ptr")
    return int(ptr.value or 0), tuple(int(d) for d in dims)


def oz2_int8_gemm(A, B, C_, batch, Mp, Np, Kp, stream=None) -> None:
    import torch
    _check(load().oz2_int8_gemm(_dev(A, torch.int8), _dev(B, torch.int8), _dev(C_, torch.int32),
                                int(batch), Mp, Np, Kp, _stream(stream)), "oz2_int8_gemm")


def oz2_mfma_probe(random_operands: bool, seconds: float = 0.25):
    """(1e12 INT8 op/s of the matrix cores alone, compute units, nominal clock in MHz)."""
    tops, cus, mhz = C.c_double(), C.c_int(), C.c_int()
    _check(load().oz2_mfma_probe(int(bool(random_operands)), float(seconds), C.byref(tops), C.byref(cus),
                                 C.byref(mhz)), "oz2_mfma_probe")
    return float(tops.value), int(cus.value), int(mhz.value)


def oz2_set_int32_products(on: bool) -> None:
    load().oz2_set_int32_products(int(bool(on)))


def oz2_set_overlap(on: bool) -> None:
    load().oz2_set_overlap(int(bool(on)))


def oz2_set_small_conversion(on: bool) -> None:
    load().oz2_set_small_conversion(int(bool(on)))


def oz2_set_profiling(on: bool) -> None:
    load().oz2_set_profiling(int(bool(on)))


def oz2_last_stage_times_ms():
    out = (C.c_float * 4)()
    _check(load().oz2_last_stage_times_ms(out), "oz2_last_stage_times_ms")
    return [float(x) for x in out]


# ------------------------------------------------------------------ contexts
def _ctx(ctx) -> C.c_void_p:
    """None (the default context), a Context, or a raw handle."""
    if ctx is None:
        return C.c_void_p(0)
    return C.c_void_p(ctx.handle if isinstance(ctx, Context) else int(ctx))


class Context:
    """Owner of an oz2_context handle (oz2_create); destroyed with the object."""

    def __init__(self):
        out = C.c_void_p(0)
        _check(load().oz2_create(C.byref(out)), "oz2_create")
        self.handle = int(out.value)

    def destroy(self) -> None:
        if self.handle:
            _check(load().oz2_destroy(C.c_void_p(self.handle)), "oz2_destroy")
            self.handle = 0

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def oz2_create() -> Context:
    return Context()


def oz2_destroy(ctx: Context) -> None:
    ctx.destroy()


def oz2_ctx_set_option(ctx, option: int, value) -> None:
    _check(load().oz2_ctx_set_option(_ctx(ctx), int(option), int(bool(value))), "oz2_ctx_set_option")


def oz2_ctx_dgemm(ctx, opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                  stream=None) -> None:
    import torch
    _check(load().oz2_ctx_dgemm(_ctx(ctx), int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                                _dev(A, torch.float64), lda, _dev(B, torch.float64), ldb, float(beta),
                                _dev(C_, torch.float64), ldc, int(num_moduli), _stream(stream)),
           "oz2_ctx_dgemm")


def oz2_ctx_sgemm(ctx, opA, opB, accurate, m, n, k, alpha, A, lda, B, ldb, beta, C_, ldc, num_moduli,
                  stream=None) -> None:
    import torch
    _check(load().oz2_ctx_sgemm(_ctx(ctx), int(opA), int(opB), int(bool(accurate)), m, n, k, float(alpha),
                                _dev(A, torch.float32), lda, _dev(B, torch.float32), ldb, float(beta),
                                _dev(C_, torch.float32), ldc, int(num_moduli), _stream(stream)),
           "oz2_ctx_sgemm")


def oz2_ctx_dgemm_prepared(ctx, left: Operand, right: Operand, alpha, beta, C_, ldc, stream=None) -> None:
    import torch
    _check(load().oz2_ctx_dgemm_prepared(_ctx(ctx), C.c_void_p(left.handle), C.c_void_p(right.handle),
                                         float(alpha), float(beta), _dev(C_, torch.float64), ldc,
                                         _stream(stream)), "oz2_ctx_dgemm_prepared")


def oz2_ctx_sgemm_prepared(ctx, left: Operand, right: Operand, alpha, beta, C_, ldc, stream=None) -> None:
    import torch
    _check(load().oz2_ctx_sgemm_prepared(_ctx(ctx), C.c_void_p(left.handle), C.c_void_p(right.handle),
                                         float(alpha), float(beta), _dev(C_, torch.float32), ldc,
                                         _stream(stream)), "oz2_ctx_sgemm_prepared")


def oz2_ctx_workspace_bytes(ctx, m, n, k, num_moduli) -> int:
    return int(load().oz2_ctx_workspace_bytes(_ctx(ctx), m, n, k, int(num_moduli)))


def oz2_ctx_workspace_min_bytes(ctx, m, n, k, num_moduli) -> int:
    return int(load().oz2_ctx_workspace_min_bytes(_ctx(ctx), m, n, k, int(num_moduli)))


def oz2_ctx_set_workspace(ctx, buf) -> None:
    if buf is None:
        _check(load().oz2_ctx_set_workspace(_ctx(ctx), C.c_void_p(0), 0), "oz2_ctx_set_workspace")
    else:
        _check(load().oz2_ctx_set_workspace(_ctx(ctx), _dev(buf), buf.numel() * buf.element_size()),
               "oz2_ctx_set_workspace")


def oz2_ctx_set_workspace_limit(ctx, nbytes: int) -> None:
    _check(load().oz2_ctx_set_workspace_limit(_ctx(ctx), int(nbytes)), "oz2_ctx_set_workspace_limit")


def oz2_ctx_plan_panels(ctx, m, n, k, num_moduli, workspace_bytes) -> Tuple[int, int, int]:
    pr, pc, cnt = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load().oz2_ctx_plan_panels(_ctx(ctx), m, n, k, int(num_moduli), int(workspace_bytes), C.byref(pr),
                                      C.byref(pc), C.byref(cnt)), "oz2_ctx_plan_panels")
    return int(pr.value), int(pc.value), int(cnt.value)


def oz2_ctx_last_panels(ctx) -> Tuple[int, int, int]:
    pr, pc, cnt = C.c_int64(), C.c_int64(), C.c_int64()
    _check(load().oz2_ctx_last_panels(_ctx(ctx), C.byref(pr), C.byref(pc), C.byref(cnt)), "oz2_ctx_last_panels")
    return int(pr.value), int(pc.value), int(cnt.value)


def oz2_ctx_last_gemm_launches(ctx) -> int:
    cnt = C.c_int64()
    _check(load().oz2_ctx_last_gemm_launches(_ctx(ctx), C.byref(cnt)), "oz2_ctx_last_gemm_launches")
    return int(cnt.value)


def oz2_last_gemm_launches() -> int:
    return oz2_ctx_last_gemm_launches(None)


def oz2_ctx_release(ctx) -> None:
    _check(load().oz2_ctx_release(_ctx(ctx)), "oz2_ctx_release")


def oz2_ctx_stage_ptr(ctx, stage: int) -> Tuple[int, Tuple[int, int, int, int]]:
    ptr = C.c_void_p(0)
    dims = (C.c_int64 * 4)()
    _check(load().oz2_ctx_stage_ptr(_ctx(ctx), int(stage), C.byref(ptr), dims), "oz2_ctx_stage_ptr")
    return int(ptr.value or 0), tuple(int(d) for d in dims)


def oz2_ctx_last_stage_times_ms(ctx):
    out = (C.c_float * 4)()
    _check(load().oz2_ctx_last_stage_times_ms(_ctx(ctx), out), "oz2_ctx_last_stage_times_ms")
    return [float(x) for x in out]


# ------------------------------------------------------------------ conveniences (no arithmetic)
def stage_tensor(stage: int, copy: bool = True, ctx=None, sync: bool = True):
    """A stage buffer of the last call (of `ctx`; None: the default context) as a torch tensor.
    Synchronises the device first unless sync=False.  With copy=False the tensor aliases the
    library's workspace and is valid until the next call."""
    import torch
    ptr, dims = oz2_ctx_stage_ptr(ctx, stage)
    if sync:
        torch.cuda.synchronize()
    torch.cuda.synchronize()
    if stage in (OZ2_STAGE_SHIFT_A, OZ2_STAGE_SHIFT_B):
        shape, dtype = (dims[0],), torch.int32
    elif stage in (OZ2_STAGE_RES_A, OZ2_STAGE_RES_B):
        shape, dtype = (dims[0], dims[2] // 64, dims[1], 64), torch.int8     # K-blocked
    elif stage == OZ2_STAGE_U:
        shape, dtype = dims[:3], torch.uint8
    else:
        shape, dtype = dims[:3], torch.int32
    typestr = {torch.int32: "<i4", torch.int8: "|i1", torch.uint8: "|u1"}[dtype]
    view = torch.as_tensor(_DeviceView(ptr, tuple(shape), typestr), device="cuda")
    return view.clone() if copy else view


class _DeviceView:
    """Zero-copy description of library-owned device memory for torch.as_tensor."""

    def __init__(self, ptr: int, shape, typestr: str):
        self.__cuda_array_interface__ = dict(shape=shape, typestr=typestr, data=(ptr, False),
                                             version=2, strides=None)


def unblock_slices(t):
    """[N][K/64][R][64] (the library's K-blocked slice layout) -> [N][R][K]."""
    n, kb, r, w = t.shape
    return t.permute(0, 2, 1, 3).reshape(n, r, kb * w)


def block_slices(t):
    """[N][R][K] -> [N][K/64][R][64], K a multiple of 64."""
    n, r, k = t.shape
    return t.reshape(n, r, k // 64, 64).permute(0, 2, 1, 3).contiguous()


def _ld(t):
    """(is a transposed view?, leading dimension of the stored matrix) of a 2-D tensor that is
    row-major or the transposed view of a row-major one."""
    r, c = t.shape
    if c == 1 or t.stride(1) == 1:
        return False, (t.stride(0) if r > 1 else max(c, 1))
    if r == 1 or t.stride(0) == 1:
        return True, (t.stride(1) if c > 1 else max(r, 1))
    raise ValueError("row-major operands, or transposed views of them, expected")


def matmul(A, B, num_moduli: int, alpha: float = 1.0, beta: float = 0.0, out=None, stream=None,
           accurate: bool = False, ctx=None):
    """C = alpha * A @ B + beta * out for device tensors that are row-major or transposed views
    (`X.t()`) of row-major ones, via oz2_ctx_dgemm / oz2_ctx_sgemm (ctx None: the default context)."""
    import torch
    if A.dim() != 2 or B.dim() != 2 or A.shape[1] != B.shape[0] or A.dtype != B.dtype:
        raise ValueError("A (m x k) and B (k x n) of one dtype expected")
    m, k = A.shape
    n = B.shape[1]
    ta, lda = _ld(A)
    tb, ldb = _ld(B)
    if out is None:
        if beta != 0.0:
            raise ValueError("beta != 0 needs `out`")
        out = torch.empty((m, n), dtype=A.dtype, device=A.device)
    if out.stride(1) != 1 and n > 1:
        raise ValueError("row-major `out` expected")
    ldc = out.stride(0) if m > 1 else max(n, 1)
    fn = oz2_ctx_dgemm if A.dtype == torch.float64 else oz2_ctx_sgemm
    fn(ctx, OZ2_OP_T if ta else OZ2_OP_N, OZ2_OP_T if tb else OZ2_OP_N, accurate, m, n, k, alpha, A, lda, B, ldb,
       beta, out, ldc, num_moduli, stream)
    return out
