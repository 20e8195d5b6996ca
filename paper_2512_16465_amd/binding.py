"""ctypes binding of libgemm's C ABI (include/gemm.h): same names, argument marshalling only.

Every step of a GEMM call runs in the HIP kernels of libgemm.so.  There is no fallback: if the
shared library is missing or does not load, the first use raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgemm.so")

# enums of include/gemm.h
GEMM_OK, GEMM_ERR_INVALID_ARG, GEMM_ERR_UNSUPPORTED, GEMM_ERR_ALLOC, GEMM_ERR_HIP, GEMM_ERR_SCRATCH_LIMIT = 0, 1, 2, 3, 4, 5
GEMM_NOALLOC_SCRATCH_BYTES = 32 << 20
GEMM_OP_N, GEMM_OP_T = 0, 1
GEMM_F32, GEMM_F16, GEMM_BF16 = 0, 1, 2
GEMM_ACT_NONE, GEMM_ACT_GELU_ERF, GEMM_ACT_RELU, GEMM_ACT_SILU, GEMM_ACT_GELU_TANH = 0, 1, 2, 3, 4
GEMM_KERNEL_AUTO, GEMM_KERNEL_GENERAL, GEMM_KERNEL_MFMA_TILE, GEMM_KERNEL_SKINNY = 0, 1, 2, 3
GEMM_MEMORY_BOUND, GEMM_MIDDLE_ZONE, GEMM_COMPUTE_BOUND = 0, 1, 2

EXPORTED_SYMBOLS = (
    "gemm_create", "gemm_run", "gemm_run_batched", "gemm_destroy", "gemm_status_string",
    "gemm_set_plan", "gemm_get_last_plan", "gemm_variant_name", "gemm_plan_query",
    "gemm_reserve_workspace", "gemm_workspace_size", "gemm_run_noalloc", "gemm_roofline_class",
)


class gemm_epilogue_t(ctypes.Structure):
    _fields_ = [("out_dtype", ctypes.c_int), ("bias", ctypes.c_void_p),
                ("bias_dtype", ctypes.c_int), ("act", ctypes.c_int)]


class gemm_plan_t(ctypes.Structure):
    _fields_ = [("kernel", ctypes.c_int), ("variant", ctypes.c_int32), ("split_k", ctypes.c_int32)]


class GemmError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {gemm_status_string(status)} (status {status})")
        self.status = status


_lib = None


def load_library() -> ctypes.CDLL:
    """Loads libgemm.so from the package directory; raises if it is not there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2512_16465_amd.build` "
            "(there is no non-HIP path)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    lib.gemm_create.restype = ctypes.c_int
    lib.gemm_create.argtypes = [ctypes.POINTER(vp)]
    lib.gemm_destroy.restype = ctypes.c_int
    lib.gemm_destroy.argtypes = [vp]
    lib.gemm_status_string.restype = ctypes.c_char_p
    lib.gemm_status_string.argtypes = [ctypes.c_int]
    lib.gemm_run.restype = ctypes.c_int
    lib.gemm_run.argtypes = [vp, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                             ctypes.c_float, vp, i64, vp, i64, ctypes.c_float, vp, i64,
                             ctypes.POINTER(gemm_epilogue_t), vp]
    lib.gemm_run_noalloc.restype = ctypes.c_int
    lib.gemm_run_noalloc.argtypes = lib.gemm_run.argtypes
    lib.gemm_run_batched.restype = ctypes.c_int
    lib.gemm_run_batched.argtypes = [vp, i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                     ctypes.c_float, vp, i64, i64, vp, i64, i64, ctypes.c_float, vp, i64, i64,
                                     ctypes.POINTER(gemm_epilogue_t), vp]
    lib.gemm_set_plan.restype = ctypes.c_int
    lib.gemm_set_plan.argtypes = [vp, ctypes.POINTER(gemm_plan_t)]
    lib.gemm_get_last_plan.restype = ctypes.c_int
    lib.gemm_get_last_plan.argtypes = [vp, ctypes.POINTER(gemm_plan_t)]
    lib.gemm_plan_query.restype = ctypes.c_int
    lib.gemm_plan_query.argtypes = [ctypes.c_int32, i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                    i64, i64, i64, ctypes.POINTER(gemm_plan_t)]
    lib.gemm_reserve_workspace.restype = ctypes.c_int
    lib.gemm_reserve_workspace.argtypes = [vp, ctypes.c_size_t]
    lib.gemm_workspace_size.restype = ctypes.c_int
    lib.gemm_workspace_size.argtypes = [vp, ctypes.POINTER(ctypes.c_size_t)]
    lib.gemm_roofline_class.restype = ctypes.c_int
    lib.gemm_roofline_class.argtypes = [i64, i64, i64, i64, ctypes.c_int, ctypes.c_int, ctypes.c_int32, ctypes.c_int32, ctypes.c_int,
                                        ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_double)]
    lib.gemm_variant_name.restype = ctypes.c_char_p
    lib.gemm_variant_name.argtypes = [ctypes.c_int, ctypes.c_int32]
    _lib = lib
    return lib


def gemm_status_string(status: int) -> str:
    return load_library().gemm_status_string(int(status)).decode()


def gemm_create() -> int:
    """Returns an opaque handle (an integer address) bound to the current HIP device."""
    h = ctypes.c_void_p()
    st = load_library().gemm_create(ctypes.byref(h))
    if st != GEMM_OK:
        raise GemmError(st, "gemm_create")
    return h.value


def gemm_destroy(handle: int) -> None:
    st = load_library().gemm_destroy(ctypes.c_void_p(handle))
    if st != GEMM_OK:
        raise GemmError(st, "gemm_destroy")


def gemm_reserve_workspace(handle: int, nbytes: int, check: bool = True) -> int:
    """The caller must have synchronised the streams that used the handle."""
    st = load_library().gemm_reserve_workspace(ctypes.c_void_p(handle), ctypes.c_size_t(nbytes))
    if check and st != GEMM_OK:
        raise GemmError(st, "gemm_reserve_workspace")
    return st


def gemm_workspace_size(handle: int) -> int:
    n = ctypes.c_size_t()
    st = load_library().gemm_workspace_size(ctypes.c_void_p(handle), ctypes.byref(n))
    if st != GEMM_OK:
        raise GemmError(st, "gemm_workspace_size")
    return n.value


def gemm_run(handle: int, M: int, N: int, K: int, transA: int, transB: int, dtype: int,
             alpha: float, A: int, lda: int, B: int, ldb: int, beta: float, C: int, ldc: int,
             epilogue: Optional[gemm_epilogue_t] = None, stream: int = 0, check: bool = True) -> int:
    """A, B, C, epilogue.bias are device addresses (e.g. tensor.data_ptr()); stream is a
    hipStream_t as an integer.  Returns the status; raises GemmError unless check is False."""
    st = load_library().gemm_run(
        ctypes.c_void_p(handle), M, N, K, transA, transB, dtype, ctypes.c_float(alpha),
        ctypes.c_void_p(A), lda, ctypes.c_void_p(B), ldb, ctypes.c_float(beta),
        ctypes.c_void_p(C), ldc, ctypes.byref(epilogue) if epilogue is not None else None,
        ctypes.c_void_p(stream))
    if check and st != GEMM_OK:
        raise GemmError(st, "gemm_run")
    return st


def gemm_run_noalloc(handle: int, M: int, N: int, K: int, transA: int, transB: int, dtype: int,
                     alpha: float, A: int, lda: int, B: int, ldb: int, beta: float, C: int, ldc: int,
                     epilogue: Optional[gemm_epilogue_t] = None, stream: int = 0, check: bool = True) -> int:
    """gemm_run with the split-K scratch in the library's static device buffer: allocates nothing."""
    st = load_library().gemm_run_noalloc(
        ctypes.c_void_p(handle), M, N, K, transA, transB, dtype, ctypes.c_float(alpha),
        ctypes.c_void_p(A), lda, ctypes.c_void_p(B), ldb, ctypes.c_float(beta),
        ctypes.c_void_p(C), ldc, ctypes.byref(epilogue) if epilogue is not None else None,
        ctypes.c_void_p(stream))
    if check and st != GEMM_OK:
        raise GemmError(st, "gemm_run_noalloc")
    return st


def gemm_run_batched(handle: int, batch: int, M: int, N: int, K: int, transA: int, transB: int, dtype: int,
                     alpha: float, A: int, lda: int, strideA: int, B: int, ldb: int, strideB: int,
                     beta: float, C: int, ldc: int, strideC: int,
                     epilogue: Optional[gemm_epilogue_t] = None, stream: int = 0, check: bool = True) -> int:
    """`batch` products of one shape; matrix b of each operand starts b * stride elements after the first."""
    st = load_library().gemm_run_batched(
        ctypes.c_void_p(handle), batch, M, N, K, transA, transB, dtype, ctypes.c_float(alpha),
        ctypes.c_void_p(A), lda, strideA, ctypes.c_void_p(B), ldb, strideB, ctypes.c_float(beta),
        ctypes.c_void_p(C), ldc, strideC, ctypes.byref(epilogue) if epilogue is not None else None,
        ctypes.c_void_p(stream))
    if check and st != GEMM_OK:
        raise GemmError(st, "gemm_run_batched")
    return st


def gemm_set_plan(handle: int, kernel: int = GEMM_KERNEL_AUTO, variant: int = -1, split_k: int = 0,
                  check: bool = True) -> int:
    """kernel == GEMM_KERNEL_AUTO restores automatic choice."""
    lib = load_library()
    if kernel == GEMM_KERNEL_AUTO:
        st = lib.gemm_set_plan(ctypes.c_void_p(handle), None)
    else:
        plan = gemm_plan_t(kernel, variant, split_k)
        st = lib.gemm_set_plan(ctypes.c_void_p(handle), ctypes.byref(plan))
    if check and st != GEMM_OK:
        raise GemmError(st, "gemm_set_plan")
    return st


def gemm_get_last_plan(handle: int):
    plan = gemm_plan_t()
    st = load_library().gemm_get_last_plan(ctypes.c_void_p(handle), ctypes.byref(plan))
    if st != GEMM_OK:
        raise GemmError(st, "gemm_get_last_plan")
    return plan.kernel, plan.variant, plan.split_k


def gemm_plan_query(compute_units: int, batch: int, M: int, N: int, K: int, transA: int, transB: int, dtype: int,
                    out_dtype: int, lda: int, ldb: int, ldc: int, check: bool = True):
    """(kernel, variant, split_k) of the automatic plan for this shape; host only, needs no GPU."""
    plan = gemm_plan_t()
    st = load_library().gemm_plan_query(compute_units, batch, M, N, K, transA, transB, dtype, out_dtype, lda, ldb, ldc,
                                        ctypes.byref(plan))
    if st != GEMM_OK:
        if check:
            raise GemmError(st, "gemm_plan_query")
        return st
    return plan.kernel, plan.variant, plan.split_k


def gemm_roofline_class(batch: int, M: int, N: int, K: int, dtype: int, out_dtype: int, reads_c: bool = False,
                        bias_dtype: Optional[int] = None):
    """(class, arithmetic intensity in flop/byte) by the roofline rule of Section 4.3; host only."""
    cls, ai = ctypes.c_int(), ctypes.c_double()
    st = load_library().gemm_roofline_class(batch, M, N, K, dtype, out_dtype, int(bool(reads_c)), int(bias_dtype is not None),
                                            bias_dtype if bias_dtype is not None else 0, ctypes.byref(cls), ctypes.byref(ai))
    if st != GEMM_OK:
        raise GemmError(st, "gemm_roofline_class")
    return cls.value, ai.value


def gemm_variant_name(kernel: int, variant: int) -> Optional[str]:
    s = load_library().gemm_variant_name(kernel, variant)
    return s.decode() if s else None


def make_epilogue(out_dtype: int, bias: int = 0, bias_dtype: int = GEMM_F32, act: int = GEMM_ACT_NONE) -> gemm_epilogue_t:
    return gemm_epilogue_t(out_dtype, ctypes.c_void_p(bias) if bias else None, bias_dtype, act)
