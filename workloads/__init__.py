"""Seeded synthetic inputs for the GEMM workloads.

This module serves both the CPU oracle's tests and the GPU library's tests and
benchmark, and therefore holds none of the method's arithmetic: it draws random
numbers, asks torch's own converters for 16-bit bit patterns, describes the five
benchmark calls, and picks which output elements a sampled check looks at.

The five calls stand in for the categories of GEMM cases the paper's case study
names (square, transposed operand, irregular/skinny; Section 5.4, note of
Table 1); the paper's own benchmark problems are not reproduced.  "N(0, x)" is
read with x as the standard deviation throughout.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np
import torch

# element type and activation codes of the C interface (values only; no shared header)
F32, F16, BF16 = 0, 1, 2
ACT_NONE, ACT_GELU_ERF, ACT_RELU, ACT_SILU, ACT_GELU_TANH = 0, 1, 2, 3, 4

_NP_BITS = {F32: np.float32, F16: np.uint16, BF16: np.uint16}
_TORCH = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}

DEFAULT_SEED = 20251216


def itemsize(dtype: int) -> int:
    return 4 if dtype == F32 else 2


def to_bits(x: np.ndarray, dtype: int) -> np.ndarray:
    """float32 values -> storage array: float32 for F32, uint16 bit patterns (torch's
    round-to-nearest-even conversion) for F16/BF16."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F32:
        return x
    t = torch.from_numpy(x).to(_TORCH[dtype])
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_torch(bits: np.ndarray, dtype: int, device=None) -> torch.Tensor:
    """Storage array -> torch tensor of the matching dtype holding the same bits."""
    if dtype == F32:
        t = torch.from_numpy(np.ascontiguousarray(bits, dtype=np.float32))
    else:
        t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(_TORCH[dtype])
    return t.to(device) if device is not None else t


def torch_to_bits(t: torch.Tensor) -> np.ndarray:
    """torch tensor (any device) -> storage array with the same bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy().copy()
    return t.view(torch.int16).numpy().view(np.uint16).copy()


@dataclass(frozen=True)
class Config:
    """One gemm_run call and the distribution of its operands."""
    name: str
    M: int
    N: int
    K: int
    transA: int
    transB: int
    dtype: int                 # A and B
    out_dtype: int             # C (read when beta != 0, written always)
    alpha: float = 1.0
    beta: float = 0.0
    a_dist: Tuple[str, float] = ("normal", 1.0)    # ("normal", std) | ("uniform", half-width)
    b_dist: Tuple[str, float] = ("normal", 1.0)
    c_dist: Tuple[str, float] = ("normal", 1.0)
    bias_dist: Optional[Tuple[str, float]] = None  # None = no bias
    bias_dtype: int = BF16
    act: int = ACT_NONE
    lda: int = 0               # 0 = minimal
    ldb: int = 0
    ldc: int = 0
    batch: int = 1             # > 1: a strided batch, the matrices of each operand packed one after the other
    note: str = ""

    # stored shapes (rows, cols) of each operand
    def a_shape(self): return (self.K, self.M) if self.transA else (self.M, self.K)
    def b_shape(self): return (self.N, self.K) if self.transB else (self.K, self.N)
    def ld_a(self): return self.lda or self.a_shape()[1]
    def ld_b(self): return self.ldb or self.b_shape()[1]
    def ld_c(self): return self.ldc or self.N
    # elements from one matrix of the batch to the next
    def stride_a(self): return self.a_shape()[0] * self.ld_a()
    def stride_b(self): return self.b_shape()[0] * self.ld_b()
    def stride_c(self): return self.M * self.ld_c()

    def flops(self) -> int:
        return 2 * self.M * self.N * self.K * self.batch

    def algorithmic_bytes(self) -> int:
        """Each operand once; C_in only when beta != 0; bias when present."""
        n = self.M * self.K * itemsize(self.dtype) + self.K * self.N * itemsize(self.dtype)
        n += self.M * self.N * itemsize(self.out_dtype)
        if self.beta != 0.0:
            n += self.M * self.N * itemsize(self.out_dtype)
        n *= self.batch
        if self.bias_dist is not None:
            n += self.N * itemsize(self.bias_dtype)
        return n


CONFIGS: Dict[str, Config] = {
    "C1": Config("C1", 256, 256, 256, 0, 0, F32, F32,
                 a_dist=("uniform", 1.0), b_dist=("uniform", 1.0),
                 note="fp32 256^3 NN, uniform[-1,1)"),
    "C2": Config("C2", 4096, 4096, 4096, 0, 1, BF16, BF16,
                 a_dist=("normal", 1.0), b_dist=("normal", 1.0),
                 note="bf16 4096^3 NT (B stored N x K), bf16 out"),
    "C3": Config("C3", 8192, 8192, 8192, 0, 0, BF16, F32,
                 a_dist=("normal", 8192 ** -0.5), b_dist=("normal", 8192 ** -0.5),
                 note="bf16 8192^3 NN, fp32 out (headline)"),
    "C4": Config("C4", 8192, 28672, 8192, 0, 1, BF16, BF16,
                 a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 bias_dist=("normal", 0.02), bias_dtype=BF16, act=ACT_GELU_ERF,
                 note="bf16 8192x28672x8192 NT + bias + GELU, bf16 out"),
    "C5": Config("C5", 32, 16384, 16384, 0, 0, BF16, BF16, alpha=1.0, beta=1.0,
                 a_dist=("normal", 1.0), b_dist=("normal", 0.02), c_dist=("normal", 1.0),
                 note="bf16 32x16384x16384 NN skinny, alpha=beta=1, bf16 in/out"),
}

# Further shapes in the categories the paper's case study names (Section 5.4: square, transposed
# and irregular GEMM; Section 5.3 uses GEMV as its memory-bound kernel): the remaining operand
# layouts, sizes that are no multiple of any tile, a tall-and-narrow product and a single-row one.
# Reported by the bench next to the five main configurations, never as its headline.
EXTRA_CONFIGS: Dict[str, Config] = {
    "X1": Config("X1", 8192, 8192, 8192, 1, 0, BF16, BF16,
                 a_dist=("normal", 8192 ** -0.5), b_dist=("normal", 8192 ** -0.5),
                 note="bf16 8192^3 TN (A stored K x M), bf16 out"),
    "X2": Config("X2", 4096, 4096, 4096, 1, 1, F16, F16,
                 a_dist=("normal", 1.0), b_dist=("normal", 4096 ** -0.5),
                 note="fp16 4096^3 TT, fp16 out"),
    "X3": Config("X3", 8000, 8200, 8136, 0, 1, BF16, BF16,
                 a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 bias_dist=("normal", 0.5), bias_dtype=F32, act=ACT_SILU,
                 note="bf16 8000x8200x8136 NT (no multiple of a tile, partial last k slab) + bias + SiLU"),
    "X4": Config("X4", 65536, 128, 4096, 0, 0, BF16, BF16,
                 a_dist=("normal", 1.0), b_dist=("normal", 4096 ** -0.5),
                 note="bf16 65536x128x4096 NN, tall and narrow"),
    "X6": Config("X6", 4096, 4096, 4096, 0, 0, F32, F32,
                 a_dist=("normal", 1.0), b_dist=("normal", 4096 ** -0.5),
                 note="fp32 4096^3 NN on the fp32 matrix instruction"),
    "X5": Config("X5", 1, 16384, 16384, 0, 0, BF16, BF16,
                 a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 1x16384x16384 NN: a matrix-vector product through the skinny path"),
    "X7": Config("X7", 32, 16384, 16384, 0, 1, BF16, BF16, alpha=1.0, beta=1.0,
                 a_dist=("normal", 1.0), b_dist=("normal", 0.02), c_dist=("normal", 1.0),
                 note="bf16 32x16384x16384 NT skinny (B stored N x K, a weight matrix kept as [out, in]), alpha=beta=1"),
    "X8": Config("X8", 2048, 2048, 128, 0, 1, BF16, BF16, batch=32,
                 a_dist=("normal", 1.0), b_dist=("normal", 128 ** -0.5),
                 note="bf16 strided batch of 32 products 2048x2048x128 NT (the per-head score products of attention), bf16 out"),
    "X11": Config("X11", 128, 16384, 16384, 0, 1, BF16, BF16,
                  a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                  note="bf16 128x16384x16384 NT: 128 rows on a weight kept as [out, in] (between the skinny and the square regime)"),
    "X9": Config("X9", 4096, 4104, 4096, 0, 0, BF16, BF16, alpha=1.0, beta=1.0,
                 a_dist=("normal", 1.0), b_dist=("normal", 4096 ** -0.5), c_dist=("normal", 1.0),
                 bias_dist=("normal", 0.5), bias_dtype=BF16, act=ACT_RELU,
                 note="bf16 4096x4104x4096 NN + C + bias + ReLU: 16 whole tile columns and a strip of 8 columns"),
    "X10": Config("X10", 4120, 4096, 4096, 1, 1, F16, F32,
                  a_dist=("normal", 1.0), b_dist=("normal", 4096 ** -0.5),
                  note="fp16 4120x4096x4096 TT, fp32 out: 16 whole tile rows and a strip of 24 rows"),
    # matrix-vector and few-row products (the paper's memory-bound kernel, Section 5.3) on weights of 32 to 256 MiB,
    # in both layouts of the weight and in bf16 and fp32
    "G1": Config("G1", 1, 8192, 8192, 0, 1, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 1x8192x8192 NT: a matrix-vector product on a 128 MiB weight kept as [out, in]"),
    "G2": Config("G2", 8, 8192, 8192, 0, 0, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 8x8192x8192 NN: 8 rows on a 128 MiB row-major weight"),
    "G3": Config("G3", 1, 4096, 4096, 0, 0, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 1x4096x4096 NN: a matrix-vector product on a 32 MiB weight (cache resident, launch bound)"),
    "G4": Config("G4", 8, 4096, 4096, 0, 1, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 8x4096x4096 NT: 8 rows on a 32 MiB weight kept as [out, in] (cache resident, launch bound)"),
    "G7": Config("G7", 1, 4096, 4096, 0, 1, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 1x4096x4096 NT: a matrix-vector product on a 32 MiB weight kept as [out, in] (cache resident; one launch on the vector ALUs)"),
    "G8": Config("G8", 4, 28672, 8192, 0, 1, BF16, BF16, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="bf16 4x28672x8192 NT: 4 rows on a 448 MiB weight kept as [out, in] (a decoding step of four sequences)"),
    "G5": Config("G5", 1, 8192, 8192, 0, 0, F32, F32, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="fp32 1x8192x8192 NN: a matrix-vector product on a 256 MiB weight, vector ALUs"),
    "G6": Config("G6", 8, 8192, 8192, 0, 1, F32, F32, a_dist=("normal", 1.0), b_dist=("normal", 0.02),
                 note="fp32 8x8192x8192 NT: 8 rows on a 256 MiB weight kept as [out, in], vector ALUs"),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of cfg with some fields replaced (smaller shapes, padded leading dimensions ...)."""
    return replace(cfg, **kw)


def _draw(rng: np.random.Generator, dist: Tuple[str, float], shape) -> np.ndarray:
    kind, scale = dist
    if kind == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
        x *= np.float32(scale)
        return x
    if kind == "uniform":
        x = rng.random(shape, dtype=np.float32)
        x *= np.float32(2.0 * scale)
        x -= np.float32(scale)
        return x
    raise ValueError(kind)


def _store(x: np.ndarray, ld: int, dtype: int) -> np.ndarray:
    """(rows, cols) values -> 1-D storage of rows*ld elements; padding columns hold a sentinel."""
    rows, cols = x.shape
    bits = to_bits(x, dtype)
    if ld == cols:
        return bits.reshape(-1)
    pad_val = to_bits(np.full((1,), 7.0, dtype=np.float32), dtype)[0]   # never read by a correct GEMM
    full = np.full((rows, ld), pad_val, dtype=bits.dtype)
    full[:, :cols] = bits
    return full.reshape(-1)


def make_inputs(cfg: Config, seed: int = DEFAULT_SEED) -> Dict[str, Optional[np.ndarray]]:
    """Operands of cfg as 1-D storage arrays: keys A, B, C (None when beta == 0), bias (or None)."""
    out: Dict[str, Optional[np.ndarray]] = {}
    # a batch is drawn as one tall matrix: with the dense strides of Config its storage is the
    # matrices of the batch one after the other
    nb = cfg.batch
    tall = lambda shape: (nb * shape[0], shape[1])
    out["A"] = _store(_draw(np.random.default_rng([seed, 1]), cfg.a_dist, tall(cfg.a_shape())), cfg.ld_a(), cfg.dtype)
    out["B"] = _store(_draw(np.random.default_rng([seed, 2]), cfg.b_dist, tall(cfg.b_shape())), cfg.ld_b(), cfg.dtype)
    if cfg.beta != 0.0:
        out["C"] = _store(_draw(np.random.default_rng([seed, 3]), cfg.c_dist, tall((cfg.M, cfg.N))), cfg.ld_c(), cfg.out_dtype)
    else:
        out["C"] = None
    if cfg.bias_dist is not None:
        out["bias"] = to_bits(_draw(np.random.default_rng([seed, 4]), cfg.bias_dist, (cfg.N,)), cfg.bias_dtype)
    else:
        out["bias"] = None
    return out


def make_integer_inputs(cfg: Config, seed: int = DEFAULT_SEED, lo: int = -1, hi: int = 1):
    """Same shapes as make_inputs, entries i.i.d. uniform integers in [lo, hi] (exact in every
    element type).  Returns (storage dict, int64 value dict with unpadded 2-D arrays)."""
    vals = {}
    out: Dict[str, Optional[np.ndarray]] = {}

    def draw(stream, shape):
        return np.random.default_rng([seed, stream]).integers(lo, hi + 1, size=shape, dtype=np.int64)

    nb = cfg.batch                      # a batch: tall matrices, batch entry b in rows [b*rows, (b+1)*rows)
    tall = lambda shape: (nb * shape[0], shape[1])
    vals["A"] = draw(11, tall(cfg.a_shape()))
    vals["B"] = draw(12, tall(cfg.b_shape()))
    out["A"] = _store(vals["A"].astype(np.float32), cfg.ld_a(), cfg.dtype)
    out["B"] = _store(vals["B"].astype(np.float32), cfg.ld_b(), cfg.dtype)
    if cfg.beta != 0.0:
        vals["C"] = draw(13, tall((cfg.M, cfg.N)))
        out["C"] = _store(vals["C"].astype(np.float32), cfg.ld_c(), cfg.out_dtype)
    else:
        vals["C"], out["C"] = None, None
    if cfg.bias_dist is not None:
        vals["bias"] = draw(14, (cfg.N,))
        out["bias"] = to_bits(vals["bias"].astype(np.float32), cfg.bias_dtype)
    else:
        vals["bias"], out["bias"] = None, None
    return out, vals


def sample_indices(M: int, N: int, seed: int = DEFAULT_SEED, grid: int = 64):
    """A stratified sample of output elements that does not know the GPU tiling: C is cut into a
    grid x grid array of near-equal blocks (grid is reduced along a dimension shorter than it, and
    the other dimension refined so that the sample still has grid*grid strata), one element is
    drawn per block, and the four corners plus the inner neighbours of the last row and column are
    added.  Returns (rows, cols) as int64 arrays without duplicates."""
    gm = min(grid, M)
    gn = min((grid * grid) // gm, N)
    rng = np.random.default_rng([seed, 99])
    rb = np.linspace(0, M, gm + 1).astype(np.int64)
    cb = np.linspace(0, N, gn + 1).astype(np.int64)
    r = rng.integers(rb[:-1, None], rb[1:, None], size=(gm, gn))
    c = rng.integers(cb[None, :-1], cb[None, 1:], size=(gm, gn))
    rows = list(r.reshape(-1))
    cols = list(c.reshape(-1))
    for (i, j) in [(0, 0), (0, N - 1), (M - 1, 0), (M - 1, N - 1),
                   (M - 1, max(N - 2, 0)), (max(M - 2, 0), N - 1)]:
        rows.append(i)
        cols.append(j)
    pairs = np.unique(np.stack([np.asarray(rows, dtype=np.int64), np.asarray(cols, dtype=np.int64)], axis=1), axis=0)
    return pairs[:, 0].copy(), pairs[:, 1].copy()
