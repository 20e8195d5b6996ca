"""Helpers of the GPU parity tests: run one call through the C ABI binding, compare with the oracle.

Tolerances (per element, `mag` = |alpha|*sum_k|a b| + |beta*C_in| + |bias| from the oracle):
  contractual  16-bit inputs: |C - ref| <= 4e-3*mag + 1e-5;   fp32: |C - ref| <= 1e-5*mag + 1e-6
               and, for fp32, ||C - ref||_F <= 1e-5 * ||ref||_F
  diagnostic   |C - ref| <= u_out*|ref| + 1e-5*mag + tiny, u_out the unit roundoff of the type of C
               (2^-8 bf16, 2^-11 fp16, 2^-23 fp32).  It follows from fp32 accumulation (error far
               below 1e-5*mag for K <= 16384) plus one rounding of the output, and is what
               catches a dropped k-slab that the loose contractual bound would let through.
"""
from __future__ import annotations

import numpy as np
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl

U_OUT = {wl.F32: 2.0 ** -23, wl.F16: 2.0 ** -11, wl.BF16: 2.0 ** -8}


def device():
    return torch.device("cuda:0")


def stream_ptr() -> int:
    return torch.cuda.current_stream().cuda_stream


def upload(bits, dtype):
    return None if bits is None else wl.bits_to_torch(bits, dtype, device())


def nan_filled(n, dtype):
    t = torch.full((n,), float("nan"), dtype=torch.float32, device=device())
    return t.to({wl.F32: torch.float32, wl.F16: torch.float16, wl.BF16: torch.bfloat16}[dtype])


class DeviceProblem:
    """Operands of one call resident on the GPU."""

    def __init__(self, cfg: wl.Config, inputs, a_offset_elems: int = 0, b_offset_elems: int = 0):
        self.cfg = cfg
        self.inputs = inputs
        # optional misalignment: shift the operand by a few elements inside a larger allocation
        self.A = self._shifted(inputs["A"], cfg.dtype, a_offset_elems)
        self.B = self._shifted(inputs["B"], cfg.dtype, b_offset_elems)
        self.bias = upload(inputs.get("bias"), cfg.bias_dtype)
        n_c = (cfg.M - 1) * cfg.ld_c() + cfg.N if cfg.M > 0 and cfg.N > 0 else 0
        self.n_c = n_c
        if cfg.beta != 0.0:
            self.C = upload(inputs["C"], cfg.out_dtype)
        else:
            self.C = nan_filled(max(n_c, 1), cfg.out_dtype)     # write-only C: stale NaN must not leak

    @staticmethod
    def _shifted(bits, dtype, off):
        t = upload(bits, dtype)
        if off == 0:
            return t
        big = torch.empty(t.numel() + off, dtype=t.dtype, device=t.device)
        big[off:] = t
        return big[off:]

    def epilogue(self):
        cfg = self.cfg
        return lg.make_epilogue(cfg.out_dtype, self.bias.data_ptr() if self.bias is not None else 0,
                                cfg.bias_dtype, cfg.act)

    def run(self, handle, check=True):
        cfg = self.cfg
        return lg.gemm_run(handle, cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype,
                           cfg.alpha, self.A.data_ptr(), cfg.ld_a(), self.B.data_ptr(), cfg.ld_b(),
                           cfg.beta, self.C.data_ptr(), cfg.ld_c(), self.epilogue(), stream_ptr(), check=check)

    def reset_c(self):
        if self.cfg.beta != 0.0:
            self.C.copy_(upload(self.inputs["C"], self.cfg.out_dtype))
        else:
            self.C.fill_(float("nan"))

    def result_bits(self) -> np.ndarray:
        """C as a 2-D (M, ldc) array of storage bits (last row padded to ldc)."""
        torch.cuda.synchronize()
        cfg = self.cfg
        flat = wl.torch_to_bits(self.C)[: self.n_c]
        full = np.zeros(cfg.M * cfg.ld_c(), dtype=flat.dtype)
        full[: flat.size] = flat
        return full.reshape(cfg.M, cfg.ld_c())


def oracle_problem(cfg: wl.Config, inputs) -> oracle.Problem:
    return oracle.Problem(cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype,
                          inputs["A"], cfg.ld_a(), inputs["B"], cfg.ld_b(),
                          alpha=cfg.alpha, beta=cfg.beta, C=inputs.get("C"), ldc=cfg.ld_c(), c_dtype=cfg.out_dtype,
                          bias=inputs.get("bias"), bias_dtype=cfg.bias_dtype, act=cfg.act)


def decode_c(cfg: wl.Config, c_bits2d: np.ndarray) -> np.ndarray:
    """(M, ldc) storage bits -> (M, N) fp64 values."""
    vals = oracle.decode(cfg.out_dtype, np.ascontiguousarray(c_bits2d[:, : cfg.N]))
    return vals


def assert_close(cfg: wl.Config, got: np.ndarray, ref: np.ndarray, mag: np.ndarray, what: str = ""):
    """got, ref, mag: same shape (full matrix or a sample)."""
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - ref)
    if cfg.dtype == wl.F32:
        contractual = 1e-5 * mag + 1e-6
    else:
        contractual = 4e-3 * mag + 1e-5
    bad = err > contractual
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond the contractual bound; worst {err.max()} vs {contractual.flat[err.argmax()]}"
    diag = U_OUT[cfg.out_dtype] * np.abs(ref) + 1e-5 * mag + 1e-30
    if cfg.dtype == wl.F32:
        diag = contractual
    bad = err > diag
    assert not bad.any(), f"{what}: {bad.sum()} elements beyond the diagnostic bound; worst ratio {(err / diag).max()}"
    if cfg.dtype == wl.F32 and ref.size > 1:
        assert np.linalg.norm(got - ref) <= 1e-5 * np.linalg.norm(ref) + 1e-12, f"{what}: Frobenius error"


def check_full(cfg: wl.Config, inputs, c_bits2d: np.ndarray, what: str = ""):
    ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inputs), want_bounds=True)
    assert_close(cfg, decode_c(cfg, c_bits2d), ref, mag, what)


def check_sampled(cfg: wl.Config, inputs, c_bits2d: np.ndarray, seed: int, what: str = ""):
    rows, cols = wl.sample_indices(cfg.M, cfg.N, seed)
    ref, _, mag = oracle.gemm_at(oracle_problem(cfg, inputs), rows, cols)
    got = oracle.decode(cfg.out_dtype, np.ascontiguousarray(c_bits2d[rows, cols]))
    assert_close(cfg, got, ref, mag, what)
    return rows, cols


def expected_bits_exact(cfg: wl.Config, inputs) -> np.ndarray:
    """For integer-valued problems the result is unique: round the oracle's exact value once."""
    ref = oracle.gemm_full(oracle_problem(cfg, inputs))
    return oracle.encode(cfg.out_dtype, ref)


def c_bits_as_uint(cfg: wl.Config, c_bits2d: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(c_bits2d[:, : cfg.N])
    return x.view(np.uint32) if cfg.out_dtype == wl.F32 else x


class BatchedDeviceProblem:
    """A strided batch on the GPU.  `cfg` describes one product; matrix b of each operand lies
    b * stride elements into its array (a stride of 0 shares the operand), the gaps between
    matrices hold a sentinel (NaN in C when it is write-only)."""

    def __init__(self, cfg: wl.Config, batch: int, strideA: int, strideB: int, strideC: int, seed: int, integer: bool = False):
        self.cfg, self.batch = cfg, batch
        self.sA, self.sB, self.sC = strideA, strideB, strideC
        one = lambda dt, n: wl.to_bits(np.full(n, 7.0, np.float32), dt)
        a_len = (cfg.a_shape()[0] - 1) * cfg.ld_a() + cfg.a_shape()[1]
        b_len = (cfg.b_shape()[0] - 1) * cfg.ld_b() + cfg.b_shape()[1]
        c_len = (cfg.M - 1) * cfg.ld_c() + cfg.N
        A = one(cfg.dtype, (batch - 1) * strideA + a_len)
        B = one(cfg.dtype, (batch - 1) * strideB + b_len)
        C = one(cfg.out_dtype, (batch - 1) * strideC + c_len)
        bias = None
        for b in range(batch):
            inp = wl.make_integer_inputs(cfg, seed + b, -2, 2)[0] if integer else wl.make_inputs(cfg, seed + b)
            if strideA or b == 0:
                A[b * strideA: b * strideA + a_len] = inp["A"][:a_len]
            if strideB or b == 0:
                B[b * strideB: b * strideB + b_len] = inp["B"][:b_len]
            if inp["C"] is not None:
                C[b * strideC: b * strideC + c_len] = inp["C"][:c_len]
            if b == 0:
                bias = inp["bias"]
        self.host = {"A": A, "B": B, "C": C if cfg.beta != 0.0 else None, "bias": bias}
        self.A, self.B = upload(A, cfg.dtype), upload(B, cfg.dtype)
        self.bias = upload(bias, cfg.bias_dtype)
        self.C = upload(C, cfg.out_dtype) if cfg.beta != 0.0 else nan_filled(C.size, cfg.out_dtype)
        self.c_before = wl.torch_to_bits(self.C)
        self.c_len = c_len

    def run(self, handle, check=True):
        cfg = self.cfg
        epi = lg.make_epilogue(cfg.out_dtype, self.bias.data_ptr() if self.bias is not None else 0, cfg.bias_dtype, cfg.act)
        return lg.gemm_run_batched(handle, self.batch, cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, cfg.alpha,
                                   self.A.data_ptr(), cfg.ld_a(), self.sA, self.B.data_ptr(), cfg.ld_b(), self.sB,
                                   cfg.beta, self.C.data_ptr(), cfg.ld_c(), self.sC, epi, stream_ptr(), check=check)

    def oracle_problem(self) -> oracle.Problem:
        cfg, h = self.cfg, self.host
        return oracle.Problem(cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, h["A"], cfg.ld_a(), h["B"], cfg.ld_b(),
                              alpha=cfg.alpha, beta=cfg.beta, C=h["C"], ldc=cfg.ld_c(), c_dtype=cfg.out_dtype,
                              bias=h["bias"], bias_dtype=cfg.bias_dtype, act=cfg.act)

    def check(self, what: str, exact: bool = False):
        """Every matrix of the batch against the oracle; everything between the matrices untouched."""
        torch.cuda.synchronize()
        cfg = self.cfg
        after = wl.torch_to_bits(self.C)
        ref, _, mag = oracle.gemm_strided_batched(self.oracle_problem(), self.batch, self.sA, self.sB, self.sC, want_bounds=True)
        touched = np.zeros(after.size, dtype=bool)
        for b in range(self.batch):
            flat = np.zeros(cfg.M * cfg.ld_c(), dtype=after.dtype)
            flat[: self.c_len] = after[b * self.sC: b * self.sC + self.c_len]
            got = decode_c(cfg, flat.reshape(cfg.M, cfg.ld_c()))
            if exact:
                want = oracle.decode(cfg.out_dtype, oracle.encode(cfg.out_dtype, ref[b]))
                assert np.array_equal(got, want), f"{what}: matrix {b}: {np.sum(got != want)} wrong"
            else:
                assert_close(cfg, got, ref[b], mag[b], f"{what}: matrix {b}")
            idx = (b * self.sC + np.arange(cfg.M)[:, None] * cfg.ld_c() + np.arange(cfg.N)[None, :]).reshape(-1)
            touched[idx] = True
        same = after.view(np.uint8).reshape(after.size, -1) == self.c_before.view(np.uint8).reshape(after.size, -1)
        assert np.all(same.all(axis=1)[~touched]), f"{what}: memory between the matrices of C was written"
