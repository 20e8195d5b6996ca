"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times (automatic
plan, default leading dimensions): a stratified sample of 4096 output elements against the
oracle, plus properties that involve every output element without an O(MNK) reference --
integer-exact data checked by a Freivalds-style product with random sign vectors, all-ones
inputs, and run-to-run determinism."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, check_sampled, decode_c, oracle_problem

pytestmark = pytest.mark.gpu

FULL = ["C2", "C3", "C4", "C5", "X1", "X2", "X3", "X4", "X5", "X6", "X7"]
ALL = {**wl.CONFIGS, **wl.EXTRA_CONFIGS}
SKINNY = ("C5", "X5", "X7")


@pytest.fixture(scope="module")
def handle():
    h = lg.gemm_create()
    yield h
    torch.cuda.synchronize()
    lg.gemm_destroy(h)


def dense(cfg, storage, shape, ld):
    return storage.reshape(shape[0], ld)[:, : shape[1]]


@pytest.mark.parametrize("name", FULL)
def test_sampled_against_oracle(handle, name):
    cfg = ALL[name]
    print(f"{name}: generating inputs", flush=True)
    inp = wl.make_inputs(cfg)
    p = DeviceProblem(cfg, inp)
    print(f"{name}: running", flush=True)
    p.run(handle)
    bits = p.result_bits()
    kernel, variant, split = lg.gemm_get_last_plan(handle)
    print(f"{name}: plan kernel={kernel} variant={variant} split={split}; oracle on the sample", flush=True)
    expected_kernel = lg.GEMM_KERNEL_SKINNY if name in SKINNY else lg.GEMM_KERNEL_MFMA_TILE
    assert kernel == expected_kernel
    check_sampled(cfg, inp, bits, wl.DEFAULT_SEED, name)
    # same call again on the same data: same bits
    first = bits.copy()
    p.reset_c()
    p.run(handle)
    assert np.array_equal(first.view(np.uint8), p.result_bits().view(np.uint8))


@pytest.mark.parametrize("name", FULL)
def test_integer_exact_with_full_coverage(handle, name):
    """Entries in {-1, 0, 1}: every partial sum is an exact integer below 2^24, so C is unique.
    With fp32 output, C r = A (B r) and r^T C = (r^T A) B must hold EXACTLY for sign vectors r
    (int64 arithmetic on the host, O(MK + KN + MN)); each output element takes part in both."""
    cfg = wl.scaled(ALL[name], out_dtype=wl.F32, act=wl.ACT_NONE, bias_dist=None)
    inp, vals = wl.make_integer_inputs(cfg, 2024, -1, 1)
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    C = p.result_bits()[:, : cfg.N]
    Ci = np.rint(C).astype(np.int64)
    assert np.array_equal(Ci.astype(np.float32), C), "non-integer output on integer data"
    opA = vals["A"].T if cfg.transA else vals["A"]          # M x K
    opB = vals["B"].T if cfg.transB else vals["B"]          # K x N
    rng = np.random.default_rng(7)
    extra = cfg.beta * vals["C"] if cfg.beta != 0.0 else 0
    for _ in range(2):
        r = rng.choice(np.array([-1, 1], dtype=np.int64), size=cfg.N)
        want = cfg.alpha * (opA @ (opB @ r)) + (extra @ r if cfg.beta != 0.0 else 0)
        assert np.array_equal(Ci @ r, np.asarray(want, dtype=np.int64)), "row check failed"
        l = rng.choice(np.array([-1, 1], dtype=np.int64), size=cfg.M)
        want = cfg.alpha * ((l @ opA) @ opB) + (l @ extra if cfg.beta != 0.0 else 0)
        assert np.array_equal(l @ Ci, np.asarray(want, dtype=np.int64)), "column check failed"
    # and a sample against the oracle, exact
    rows, cols = wl.sample_indices(cfg.M, cfg.N, 5)
    ref, _, _ = oracle.gemm_at(oracle_problem(cfg, inp), rows, cols)
    assert np.array_equal(C[rows, cols].astype(np.float64), ref)


@pytest.mark.parametrize("name", FULL)
def test_all_ones_gives_k(handle, name):
    cfg = wl.scaled(ALL[name], act=wl.ACT_NONE, bias_dist=None)
    one = lambda shape, ld, dt: wl.to_bits(np.ones(shape[0] * ld, np.float32), dt)
    inp = {"A": one(cfg.a_shape(), cfg.ld_a(), cfg.dtype), "B": one(cfg.b_shape(), cfg.ld_b(), cfg.dtype),
           "C": one((cfg.M, cfg.N), cfg.ld_c(), cfg.out_dtype) if cfg.beta != 0.0 else None, "bias": None}
    p = DeviceProblem(cfg, inp)
    p.run(handle)
    got = decode_c(cfg, p.result_bits())
    exact = cfg.alpha * cfg.K + (cfg.beta if cfg.beta != 0.0 else 0.0)
    want = oracle.decode(cfg.out_dtype, oracle.encode(cfg.out_dtype, np.array([exact])))[0]   # e.g. 16385 -> 16384 in bf16
    assert np.all(got == want), f"{name}: {np.sum(got != want)} elements differ from {want}"
