"""gemm_run_noalloc: the entry point for callers that cannot allocate.  It must give the very bits
gemm_run gives (same kernels, the split-K partial results in the library's static device buffer
instead of the handle's workspace), on two calls in a row, the second smaller than the first, so
that whatever the first left in the shared buffer is shown not to leak into the second."""
import numpy as np
import pytest
import torch

import oracle
import paper_2512_16465_amd as lg
import workloads as wl
from gpu_harness import DeviceProblem, assert_close, decode_c, oracle_problem

pytestmark = pytest.mark.gpu


def run_noalloc(p: DeviceProblem, handle, check=True):
    cfg = p.cfg
    return lg.gemm_run_noalloc(handle, cfg.M, cfg.N, cfg.K, cfg.transA, cfg.transB, cfg.dtype, cfg.alpha,
                               p.A.data_ptr(), cfg.ld_a(), p.B.data_ptr(), cfg.ld_b(), cfg.beta, p.C.data_ptr(), cfg.ld_c(),
                               p.epilogue(), torch.cuda.current_stream().cuda_stream, check=check)


def cfg_of(M, N, K, ta, tb, out, **kw):
    return wl.Config("noalloc", M, N, K, ta, tb, wl.BF16, out, a_dist=("normal", 1.0), b_dist=("normal", 0.05), **kw)


# (plan, first call, second and smaller call); every plan splits K, i.e. uses the scratch buffer
CASES = [
    ((lg.GEMM_KERNEL_SKINNY, -1, 4), (32, 2048, 4096, 0, 0), (24, 1024, 2048, 0, 0)),          # streaming kernel, row-major B
    ((lg.GEMM_KERNEL_SKINNY, 1, 8), (17, 1536, 4096, 0, 1), (5, 512, 1024, 0, 1)),             # ... B stored N x K (the wide kernel by name: the second call would go to the one-launch kernel)
    ((lg.GEMM_KERNEL_MFMA_TILE, 5, 3), (392, 328, 1096, 0, 1), (136, 264, 520, 0, 0)),         # k slices of the 128x128 tile
    ((lg.GEMM_KERNEL_MFMA_TILE, 10, 4), (520, 776, 4096, 0, 0), (256, 264, 2048, 1, 0)),       # split tiles of the 256x256 tile
    ((lg.GEMM_KERNEL_AUTO, -1, 0), (48, 4096, 4096, 0, 1), (33, 1024, 2048, 0, 0)),            # whatever the library picks
]


@pytest.mark.parametrize("plan,first,second", CASES)
def test_noalloc_matches_gemm_run_twice_in_a_row(plan, first, second):
    h = lg.gemm_create()
    try:
        lg.gemm_set_plan(h, *plan)
        for i, shape in enumerate((first, second)):
            cfg = cfg_of(*shape, wl.BF16 if i == 0 else wl.F32, alpha=1.0, beta=0.5, c_dist=("normal", 1.0),
                         bias_dist=("normal", 0.1), bias_dtype=wl.BF16, act=wl.ACT_GELU_ERF)
            inputs = wl.make_inputs(cfg, 700 + i)
            p_ref, p_new = DeviceProblem(cfg, inputs), DeviceProblem(cfg, inputs)
            before = lg.gemm_workspace_size(h)
            run_noalloc(p_new, h)
            assert lg.gemm_workspace_size(h) == before, "the no-alloc call touched the handle's workspace"
            plan_new = lg.gemm_get_last_plan(h)
            p_ref.run(h)
            assert lg.gemm_get_last_plan(h) == plan_new
            assert plan_new[2] > 1, "the case was meant to use the scratch buffer"
            torch.cuda.synchronize()
            got, want = p_new.result_bits(), p_ref.result_bits()
            assert np.array_equal(got, want), f"call {i}: {np.sum(got != want)} elements differ from gemm_run"
            ref, _, mag = oracle.gemm_full(oracle_problem(cfg, inputs), want_bounds=True)
            assert_close(cfg, decode_c(cfg, got), ref, mag, f"noalloc call {i}")
    finally:
        torch.cuda.synchronize()
        lg.gemm_destroy(h)


def test_noalloc_rejects_what_does_not_fit_and_leaves_c_alone():
    h = lg.gemm_create()
    try:
        cfg = cfg_of(1024, 1024, 1024, 0, 0, wl.F32)
        p = DeviceProblem(cfg, wl.make_inputs(cfg, 5))
        before = p.result_bits().copy()
        lg.gemm_set_plan(h, lg.GEMM_KERNEL_MFMA_TILE, 5, 16)           # 16 slices of 4 MiB: twice the static buffer
        assert run_noalloc(p, h, check=False) == lg.GEMM_ERR_SCRATCH_LIMIT
        torch.cuda.synchronize()
        assert np.array_equal(p.result_bits().view(np.uint32), before.view(np.uint32))
        assert "scratch" in lg.gemm_status_string(lg.GEMM_ERR_SCRATCH_LIMIT)
        lg.gemm_set_plan(h, lg.GEMM_KERNEL_MFMA_TILE, 5, 8)            # 8 slices: exactly the 32 MiB it holds
        assert run_noalloc(p, h) == lg.GEMM_OK
        assert lg.gemm_workspace_size(h) == 0
        ref, _, mag = oracle.gemm_full(oracle_problem(cfg, p.inputs), want_bounds=True)
        assert_close(cfg, decode_c(cfg, p.result_bits()), ref, mag, "noalloc at the limit")
        # a plan without a split needs no scratch at all
        lg.gemm_set_plan(h)
        big = cfg_of(2048, 2048, 512, 0, 1, wl.BF16)
        q = DeviceProblem(big, wl.make_inputs(big, 6))
        assert run_noalloc(q, h) == lg.GEMM_OK
        ref, _, mag = oracle.gemm_full(oracle_problem(big, q.inputs), want_bounds=True)
        assert_close(big, decode_c(big, q.result_bits()), ref, mag, "noalloc without a split")
    finally:
        torch.cuda.synchronize()
        lg.gemm_destroy(h)
