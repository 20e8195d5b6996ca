"""Python face of the CPU oracle (``gemm_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
import this package; the GPU library never does, and this package never imports
the GPU library.  It marshals numpy arrays into the C oracle and nothing else:
all arithmetic lives in ``gemm_oracle.c``.

Arrays of 16-bit floats travel as ``numpy.uint16`` bit patterns, fp32 as
``numpy.float32`` (or ``uint32`` bit patterns).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gemm_oracle.c")
_LIB = os.path.join(_HERE, "libgemm_oracle.so")

F32, F16, BF16 = 0, 1, 2
ACT_NONE, ACT_GELU_ERF, ACT_RELU, ACT_SILU, ACT_GELU_TANH = 0, 1, 2, 3, 4

_ITEMSIZE = {F32: 4, F16: 2, BF16: 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc; returns the path of the shared object."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Problem(ctypes.Structure):
    _fields_ = [
        ("M", ctypes.c_int64), ("N", ctypes.c_int64), ("K", ctypes.c_int64),
        ("transA", ctypes.c_int32), ("transB", ctypes.c_int32),
        ("ab_dtype", ctypes.c_int32), ("c_dtype", ctypes.c_int32),
        ("bias_dtype", ctypes.c_int32), ("act", ctypes.c_int32),
        ("alpha", ctypes.c_double), ("beta", ctypes.c_double),
        ("A", ctypes.c_void_p), ("lda", ctypes.c_int64),
        ("B", ctypes.c_void_p), ("ldb", ctypes.c_int64),
        ("C", ctypes.c_void_p), ("ldc", ctypes.c_int64),
        ("bias", ctypes.c_void_p),
    ]


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int64)
        pp = ctypes.POINTER(_Problem)
        lib.oracle_decode.restype = ctypes.c_double
        lib.oracle_decode.argtypes = [ctypes.c_int, ctypes.c_uint32]
        lib.oracle_encode.restype = ctypes.c_uint32
        lib.oracle_encode.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.oracle_decode_array.restype = None
        lib.oracle_decode_array.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_int64, dp]
        lib.oracle_encode_array.restype = None
        lib.oracle_encode_array.argtypes = [ctypes.c_int, dp, ctypes.c_int64, ctypes.c_void_p]
        lib.oracle_gelu_erf.restype = ctypes.c_double
        lib.oracle_gelu_erf.argtypes = [ctypes.c_double]
        lib.oracle_act.restype = ctypes.c_double
        lib.oracle_act.argtypes = [ctypes.c_int, ctypes.c_double]
        lib.oracle_num_threads.restype = ctypes.c_int
        lib.oracle_num_threads.argtypes = []
        lib.oracle_gemm_full.restype = ctypes.c_int
        lib.oracle_gemm_full.argtypes = [pp, dp, dp, dp]
        lib.oracle_gemm_at.restype = ctypes.c_int
        lib.oracle_gemm_at.argtypes = [pp, ip, ip, ctypes.c_int64, dp, dp, dp]
        lib.oracle_gemm_rows.restype = ctypes.c_int
        lib.oracle_gemm_rows.argtypes = [pp, ctypes.c_int64, ctypes.c_int64, dp]
        _lib = lib
    return _lib


def _as_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """Accept float32/uint32 for F32 and uint16 for the 16-bit types; return a C-contiguous view."""
    x = np.ascontiguousarray(x)
    if x.dtype.itemsize != _ITEMSIZE[dtype]:
        raise TypeError(f"array of {x.dtype} cannot hold element type code {dtype}")
    return x


def _dptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


@dataclass
class Problem:
    """One GEMM call as the oracle sees it (host arrays of bit patterns, row-major storage)."""
    M: int
    N: int
    K: int
    transA: int
    transB: int
    ab_dtype: int
    A: np.ndarray
    lda: int
    B: np.ndarray
    ldb: int
    alpha: float = 1.0
    beta: float = 0.0
    C: Optional[np.ndarray] = None
    ldc: int = 0
    c_dtype: int = F32
    bias: Optional[np.ndarray] = None
    bias_dtype: int = F32
    act: int = ACT_NONE

    def _c(self):
        keep = []
        p = _Problem()
        p.M, p.N, p.K = self.M, self.N, self.K
        p.transA, p.transB = int(self.transA), int(self.transB)
        p.ab_dtype, p.c_dtype, p.bias_dtype, p.act = self.ab_dtype, self.c_dtype, self.bias_dtype, self.act
        # alpha and beta reach the GPU as binary32: widen exactly that value
        p.alpha, p.beta = float(np.float32(self.alpha)), float(np.float32(self.beta))
        a = _as_bits(self.A, self.ab_dtype); keep.append(a)
        b = _as_bits(self.B, self.ab_dtype); keep.append(b)
        a_rows = self.K if self.transA else self.M
        b_rows = self.N if self.transB else self.K
        a_cols = self.M if self.transA else self.K
        b_cols = self.K if self.transB else self.N
        if self.lda < a_cols or self.ldb < b_cols:
            raise ValueError("leading dimension smaller than the stored row length")
        if a.size < (a_rows - 1) * self.lda + a_cols and a_rows > 0 and a_cols > 0:
            raise ValueError("A array too small for M, K, lda")
        if b.size < (b_rows - 1) * self.ldb + b_cols and b_rows > 0 and b_cols > 0:
            raise ValueError("B array too small for K, N, ldb")
        p.A, p.lda = a.ctypes.data, self.lda
        p.B, p.ldb = b.ctypes.data, self.ldb
        if self.C is not None:
            c = _as_bits(self.C, self.c_dtype); keep.append(c)
            if self.ldc < self.N or (self.M > 0 and c.size < (self.M - 1) * self.ldc + self.N):
                raise ValueError("C array too small for M, N, ldc")
            p.C, p.ldc = c.ctypes.data, self.ldc
        else:
            p.C, p.ldc = None, max(self.ldc, self.N)
        if self.bias is not None:
            bb = _as_bits(self.bias, self.bias_dtype); keep.append(bb)
            if bb.size < self.N:
                raise ValueError("bias shorter than N")
            p.bias = bb.ctypes.data
        else:
            p.bias = None
        return p, keep


def decode(dtype: int, bits: np.ndarray) -> np.ndarray:
    """Bit patterns -> exact fp64 values."""
    b = _as_bits(bits, dtype)
    out = np.empty(b.size, dtype=np.float64)
    _load().oracle_decode_array(dtype, b.ctypes.data, b.size, _dptr(out))
    return out.reshape(b.shape)


def encode(dtype: int, values: np.ndarray) -> np.ndarray:
    """fp64 values -> nearest representable bit patterns (ties to even)."""
    v = np.ascontiguousarray(values, dtype=np.float64)
    out = np.empty(v.size, dtype=np.uint32 if dtype == F32 else np.uint16)
    _load().oracle_encode_array(dtype, _dptr(v), v.size, out.ctypes.data)
    return out.reshape(v.shape)


def gelu_erf(x: float) -> float:
    return float(_load().oracle_gelu_erf(float(x)))


def act(code: int, x: float) -> float:
    """The activation `code` (ACT_*) applied to one value."""
    return float(_load().oracle_act(int(code), float(x)))


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def gemm_full(p: Problem, want_bounds: bool = False):
    """All M*N reference values (fp64).  With want_bounds also sum_k|a b| and the bound magnitude."""
    cp, keep = p._c()
    ref = np.empty((p.M, p.N), dtype=np.float64)
    sa = np.empty((p.M, p.N), dtype=np.float64) if want_bounds else None
    mag = np.empty((p.M, p.N), dtype=np.float64) if want_bounds else None
    rc = _load().oracle_gemm_full(ctypes.byref(cp), _dptr(ref), _dptr(sa), _dptr(mag))
    del keep
    if rc != 0:
        raise ValueError("oracle rejected the problem")
    return (ref, sa, mag) if want_bounds else ref


def gemm_at(p: Problem, rows: np.ndarray, cols: np.ndarray):
    """Reference values, sum_k|a b| and bound magnitude at the listed (row, col) pairs."""
    cp, keep = p._c()
    r = np.ascontiguousarray(rows, dtype=np.int64)
    c = np.ascontiguousarray(cols, dtype=np.int64)
    if r.shape != c.shape:
        raise ValueError("rows and cols differ in length")
    ref = np.empty(r.size, dtype=np.float64)
    sa = np.empty(r.size, dtype=np.float64)
    mag = np.empty(r.size, dtype=np.float64)
    ip = ctypes.POINTER(ctypes.c_int64)
    rc = _load().oracle_gemm_at(ctypes.byref(cp), r.ctypes.data_as(ip), c.ctypes.data_as(ip), r.size,
                                _dptr(ref), _dptr(sa), _dptr(mag))
    del keep
    if rc != 0:
        raise ValueError("oracle rejected the problem or an index")
    return ref, sa, mag


def gemm_rows(p: Problem, row0: int, nrows: int) -> np.ndarray:
    """Reference values for rows [row0, row0+nrows), all columns."""
    cp, keep = p._c()
    ref = np.empty((nrows, p.N), dtype=np.float64)
    rc = _load().oracle_gemm_rows(ctypes.byref(cp), row0, nrows, _dptr(ref))
    del keep
    if rc != 0:
        raise ValueError("oracle rejected the problem")
    return ref


def gemm_strided_batched(p: Problem, batch: int, strideA: int, strideB: int, strideC: int, want_bounds: bool = False):
    """A strided batch by its definition: problem b is `p` with every matrix taken b * stride
    elements further into its array (bias is shared).  Returns arrays of shape (batch, M, N):
    the reference values, and with want_bounds also sum_k|a b| and the bound magnitude."""
    outs = []
    for b in range(batch):
        q = replace(p, A=p.A[b * strideA:], B=p.B[b * strideB:], C=None if p.C is None else p.C[b * strideC:])
        outs.append(gemm_full(q, want_bounds))
    if want_bounds:
        return tuple(np.stack([o[i] for o in outs]) for i in range(3))
    return np.stack(outs)
