"""CPU-only checks of the seeded input generators and of the sampling of output elements."""
import numpy as np

import oracle
import workloads as wl


def test_configs_match_the_stated_shapes():
    c = wl.CONFIGS
    assert (c["C1"].M, c["C1"].N, c["C1"].K, c["C1"].dtype, c["C1"].transB) == (256, 256, 256, wl.F32, 0)
    assert (c["C2"].M, c["C2"].transA, c["C2"].transB, c["C2"].out_dtype) == (4096, 0, 1, wl.BF16)
    assert (c["C3"].K, c["C3"].transB, c["C3"].out_dtype) == (8192, 0, wl.F32)
    assert (c["C4"].M, c["C4"].N, c["C4"].K, c["C4"].act) == (8192, 28672, 8192, wl.ACT_GELU_ERF)
    assert (c["C5"].M, c["C5"].N, c["C5"].K, c["C5"].beta) == (32, 16384, 16384, 1.0)
    assert c["C3"].flops() == 1099511627776 and c["C3"].algorithmic_bytes() == 536870912
    assert c["C5"].algorithmic_bytes() == 540016640
    assert c["C2"].algorithmic_bytes() == 100663296
    assert c["C4"].algorithmic_bytes() == 1073799168


def test_generators_are_seeded_and_have_the_stated_distributions():
    cfg = wl.scaled(wl.CONFIGS["C4"], M=96, N=160, K=512)
    a = wl.make_inputs(cfg, 7)
    b = wl.make_inputs(cfg, 7)
    c = wl.make_inputs(cfg, 8)
    for k in ("A", "B", "bias"):
        assert np.array_equal(a[k], b[k]) and not np.array_equal(a[k], c[k])
    assert a["C"] is None
    A = oracle.decode(wl.BF16, a["A"])
    B = oracle.decode(wl.BF16, a["B"])
    assert A.size == 96 * 512 and B.size == 160 * 512
    assert abs(A.std() - 1.0) < 0.02 and abs(B.std() - 0.02) < 0.0005 and abs(A.mean()) < 0.02
    u = wl.make_inputs(wl.CONFIGS["C1"], 3)["A"]
    assert u.dtype == np.float32 and u.min() >= -1.0 and u.max() < 1.0 and abs(u.mean()) < 0.02


def test_padded_leading_dimensions_keep_values():
    cfg = wl.scaled(wl.CONFIGS["C2"], M=8, N=12, K=16)
    padded = wl.scaled(cfg, lda=24, ldb=40)
    x, y = wl.make_inputs(cfg, 1), wl.make_inputs(padded, 1)
    assert np.array_equal(x["A"].reshape(8, 16), y["A"].reshape(8, 24)[:, :16])
    assert np.array_equal(x["B"].reshape(12, 16), y["B"].reshape(12, 40)[:, :16])


def test_integer_inputs_are_exact():
    cfg = wl.scaled(wl.CONFIGS["C5"], M=4, N=24, K=40)
    st, vals = wl.make_integer_inputs(cfg, 5, -2, 2)
    assert np.array_equal(oracle.decode(wl.BF16, st["A"]).reshape(4, 40), vals["A"].astype(float))
    assert np.array_equal(oracle.decode(wl.BF16, st["C"]).reshape(4, 24), vals["C"].astype(float))
    assert set(np.unique(vals["B"])) <= {-2, -1, 0, 1, 2}


def test_sample_covers_every_block_and_the_corners():
    for (M, N) in [(8192, 8192), (8192, 28672), (32, 16384), (256, 256), (5, 3)]:
        r, c = wl.sample_indices(M, N, 1)
        assert r.min() >= 0 and r.max() == M - 1 and c.min() >= 0 and c.max() == N - 1
        pairs = set(zip(r.tolist(), c.tolist()))
        assert len(pairs) == len(r)
        for p in [(0, 0), (0, N - 1), (M - 1, 0), (M - 1, N - 1)]:
            assert p in pairs
        if M * N >= 4096:
            assert 4096 <= len(r) <= 4096 + 6
            gm = min(64, M)
            gn = 4096 // gm
            blocks = set((int(i * gm // M), int(j * gn // N)) for i, j in pairs)
            assert len(blocks) == gm * gn      # every stratum holds a sample


def test_bits_round_trip_through_torch():
    x = np.random.default_rng(0).standard_normal(1000).astype(np.float32)
    for dt in (wl.F32, wl.F16, wl.BF16):
        bits = wl.to_bits(x, dt)
        assert np.array_equal(wl.torch_to_bits(wl.bits_to_torch(bits, dt)), bits)
