"""The generated code of the direct-to-LDS tile kernels never touches a fragment register between
its LDS read and the kernel's own wait for it (tests/asm_inflight.py explains why that can happen).

CPU only: the device side of each translation unit is compiled to assembly text and read.
"""
import concurrent.futures
import os

import pytest

from asm_inflight import check_listing, check_wide_store_data

# ---- the checker itself, on listings small enough to read ----

COPY_BEFORE_WAIT = """
_Z1kv:
	ds_read_b128 v[4:7], v1 offset:0
	v_mov_b64_e32 v[10:11], v[4:5]
	s_waitcnt lgkmcnt(0)
	v_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[12:15], a[0:3]
	s_endpgm
"""
USE_AFTER_WAIT = COPY_BEFORE_WAIT.replace("\tv_mov_b64_e32 v[10:11], v[4:5]\n", "")
COUNTED_WAIT = """
_Z1kv:
	ds_read_b128 v[4:7], v1 offset:0
	ds_read_b128 v[8:11], v1 offset:1024
	s_waitcnt lgkmcnt(1)
	v_mfma_f32_16x16x32_bf16 a[0:3], v[4:7], v[12:15], a[0:3]
	USE_OF_YOUNGER
	s_waitcnt lgkmcnt(0)
	s_endpgm
"""
ACROSS_A_LOOP = """
_Z1kv:
	ds_read_b64_tr_b16 v[2:3], v1
.LBB0_1:
	s_waitcnt vmcnt(0) lgkmcnt(0)
	v_mfma_f32_16x16x32_bf16 a[0:3], v[2:5], v[12:15], a[0:3]
	ds_read_b64_tr_b16 v[2:3], v1
	s_cbranch_scc1 .LBB0_1
	AFTER_THE_LOOP
	s_waitcnt lgkmcnt(0)
	s_endpgm
"""


def findings(text, **kw):
    return check_listing(text.splitlines(), **kw)[1]


def test_checker_flags_a_copy_placed_before_the_wait():
    f = findings(COPY_BEFORE_WAIT)
    assert len(f) == 1 and f[0][3].startswith("v_mov_b64") and ("v", 4) in f[0][2]
    assert findings(USE_AFTER_WAIT) == []


def test_checker_counts_lds_operations_in_order():
    assert findings(COUNTED_WAIT.replace("USE_OF_YOUNGER", "s_nop 0")) == []
    f = findings(COUNTED_WAIT.replace("USE_OF_YOUNGER", "v_add_u32_e32 v20, v8, v8"))
    assert len(f) == 1 and ("v", 8) in f[0][2]


def test_checker_follows_the_control_flow_graph():
    assert findings(ACROSS_A_LOOP.replace("AFTER_THE_LOOP", "s_nop 0")) == []
    # the read of the last trip is still in flight where the loop falls through
    f = findings(ACROSS_A_LOOP.replace("AFTER_THE_LOOP", "v_mov_b32_e32 v3, 0"))
    assert len(f) == 1 and f[0][2] == [("v", 3)]
    # a later LDS read may write the register again (in-order return), its address may not come from it
    assert findings(ACROSS_A_LOOP.replace("AFTER_THE_LOOP", "ds_read_b64_tr_b16 v[2:3], v1")) == []
    assert len(findings(ACROSS_A_LOOP.replace("AFTER_THE_LOOP", "ds_read_b64_tr_b16 v[6:7], v2"))) == 1


def test_checker_flags_a_write_to_store_data_right_behind_a_wide_store():
    text = """
_Z1kv:
	global_store_dwordx4 v[10:11], v[4:7], off nt
	NEXT
	s_endpgm
"""
    write = "v_lshl_add_u64 v[4:5], v[10:11], 0, s[2:3]"
    assert len(check_wide_store_data(text.replace("NEXT", write).splitlines())) == 1
    assert len(check_wide_store_data(text.replace("NEXT", "s_nop 0\n\t" + write).splitlines())) == 1
    assert len(check_wide_store_data(text.replace("NEXT", "s_mov_b32 s0, 0\n\t" + write).splitlines())) == 1
    assert check_wide_store_data(text.replace("NEXT", "s_nop 1\n\t" + write).splitlines()) == []
    assert check_wide_store_data(text.replace("NEXT", "s_nop 0\n\ts_mov_b32 s0, 0\n\t" + write).splitlines()) == []
    assert check_wide_store_data(text.replace("NEXT", "v_lshl_add_u64 v[10:11], v[10:11], 0, s[2:3]").splitlines()) == []
    assert check_wide_store_data(text.replace("x4", "x2").replace("NEXT", "v_mov_b32_e32 v4, 0").splitlines()) == []


# ---- the library's kernels ----

# every direct-to-LDS variant that the automatic plan can choose (5, 12, 10, 14, 15, 16, 17) and the older ones that
# only a forced plan reaches, with the kernel family in each unit.  Not listed: variant 8 (tile_dma_pair_kernel.hpp,
# forced plans only), where the checker, which does not know that the hot loop always leaves k steps for the edge
# loop, reports the path "hot loop, no edge step, epilogue"; its loop bounds (kt + 6 <= full_tiles, then kt < k_tiles)
# rule that path out.
CHECKED_UNITS = [
    ("tile_variant_4.hip", "tile_dma_kernel"), ("tile_variant_6.hip", "tile_dma_kernel"),
    ("tile_variant_7.hip", "tile_dma_kernel"), ("tile_variant_9.hip", "tile_dma16_kernel"),
    ("tile_variant_5.hip", "tile_dma_kernel"), ("tile_variant_12.hip", "tile_dma_kernel"),
    ("tile_variant_10.hip", "tile_dma16_kernel"), ("tile_variant_14.hip", "tile_dma16_kernel"),
    ("tile_variant_15.hip", "tile_dma16_kernel"), ("tile_variant_16.hip", "tile_dma16_kernel"),
    ("tile_variant_17.hip", "tile_shortk_kernel"),
    # the streaming kernels for B stored N x K read their ring with the same kind of assembly (wide and 16-column form)
    ("skinny_kernel.hip", "skinny_nt"),
]


@pytest.fixture(scope="module")
def listings(tmp_path_factory):
    from paper_2512_16465_amd import build
    if not os.path.exists(build.HIPCC):
        pytest.skip("no hipcc")
    out = tmp_path_factory.mktemp("asm")
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        jobs = {u: pool.submit(build.device_assembly, u, str(out / (u + ".s"))) for u, _ in CHECKED_UNITS}
        return {u: j.result() for u, j in jobs.items()}


@pytest.mark.parametrize("unit,family", CHECKED_UNITS)
def test_no_fragment_register_is_touched_before_its_wait(listings, unit, family):
    with open(listings[unit]) as f:
        kernels, found = check_listing(f, only=family)
    assert kernels >= 8, f"{unit}: expected the instantiations of {family}, found {kernels} kernels"
    assert not found, f"{unit}: {len(found)} findings, first: {found[0]}"
    with open(listings[unit]) as f:
        found = check_wide_store_data(f)
    assert not found, f"{unit}: wide store data overwritten without a wait state, first: {found[0]}"


def test_short_k_kernel_waits_count_the_operations_the_source_says(listings):
    """The short-k kernel waits for its operands by counting the wave's younger memory operations: the loads of
    the second pair of slabs (2 per slab for A, 2 more where B is requested too) and the stores of the tile before
    (8 per wave for a 16-bit C, 16 for fp32).  The immediates in the generated code are those sums:
    four slabs 2*4+NST or 2*2+NST, three slabs 4+NST or 2+NST, and NST before the second pair and for one or
    two slabs."""
    import collections
    import re
    waits, kernel = collections.defaultdict(set), None
    with open(listings["tile_variant_17.hip"]) as f:
        lines = f.read().splitlines()
    for i, line in enumerate(lines):
        m = re.match(r"^(_ZN4gemm4tile18tile_shortk_kernel\S*):", line)
        if m:
            kernel = m.group(1)
        m = re.search(r"s_waitcnt vmcnt\((\d+)\) lgkmcnt\(0\)", line)
        if m and kernel and "s_barrier" in lines[i + 1]:
            waits[kernel].add(int(m.group(1)))
    assert len(waits) == 24
    for name, seen in waits.items():
        out = int(re.search(r"ELi(\d)EEEv", name).group(1))          # last template argument: 0 fp32, 1 fp16, 2 bf16
        nst = 16 if out == 0 else 8
        assert seen == {nst + 8, nst + 4, nst + 2, nst}, (name, sorted(seen))
