"""CPU-only bounds arithmetic for the direct-to-LDS operand movers (csrc/tile_dma_kernel.hpp).

The steady state of the direct-to-LDS tile kernels advances along k with the loads' scalar offset,
which the buffer descriptor's range check does not see: the check compares only the per-lane
offset with the bytes left from the tile's first slab.  A lane that passes the check therefore
reads at  tile base + k advance + lane offset  whatever that address is.  This test restates the
movers' address arithmetic (DmaKC::init, DmaMC::init, tile_base, k_step_bytes, total_bytes) and
checks over edge shapes that every load the hardware performs stays inside the operand, for every
slab that the steady state may request (all slabs that lie wholly inside K, in any order: a rotated
walk visits all of them).  The same arithmetic without the clamp of DmaMC::init is shown to leave
the operand, so the test would notice the clamp being lost.
"""
import itertools

import numpy as np
import pytest

NT, BK = 256, 32


def mc_swizzle(k):
    return ((k & 3) << 2) ^ (((k >> 3) & 1) << 1)


def kc_line_hash(line, fold):
    return ((line ^ (line >> 3)) & 7) if fold else (line & 7)


def kc_offsets(rows_tile, ld, fold):
    """DmaKC::init: byte offset of every (load, thread) chunk from the slab's first byte."""
    cpr = BK // 8
    slots = np.arange(rows_tile * cpr)
    line = slots >> 3
    pos = (slots & 7) ^ np.array([kc_line_hash(int(l), fold) for l in line])
    chunk = (line << 3) | pos
    row, c = chunk // cpr, chunk % cpr
    return (row * ld + c * 8) * 2


def mc_offsets(rows_tile, ld, valid_rows, clamp=True):
    """DmaMC::init."""
    cpk = rows_tile // 8
    slots = np.arange(BK * cpk)
    k, cs = slots // cpk, slots % cpk
    c = cs ^ np.array([mc_swizzle(int(x)) for x in k])
    c8 = c * 8
    if clamp:
        c8 = np.where(c8 + 8 <= valid_rows, c8, valid_rows - 8)
    return (k * ld + c8) * 2


def max_overrun(kc, rows_tile, rows, K, ld, fold=False, clamp=True, slab0=0):
    """Largest number of bytes by which a performed load ends past the operand (<= 0: inside)."""
    total = ((rows - 1) * ld + K) * 2 if kc else ((K - 1) * ld + rows) * 2
    step = BK * 2 if kc else BK * ld * 2
    full_slabs = K // BK
    worst = -10 ** 18
    for first in range(0, rows, rows_tile):
        base = (first * ld * 2 if kc else first * 2) + slab0 * step
        records = total - base                      # make_rsrc(p, bytes left from the tile's first slab)
        valid = min(rows_tile, rows - first)
        off = kc_offsets(rows_tile, ld, fold) if kc else mc_offsets(rows_tile, ld, valid, clamp)
        performed = off + 16 <= min(records, 0xffffffff)     # lanes that pass the range check
        if not performed.any():
            continue
        for p in range(slab0, full_slabs):
            soff = (p - slab0) * step
            end = base + soff + off[performed] + 16
            worst = max(worst, int(end.max()) - total)
    return worst


EDGE_SHAPES = [
    # rows of the operand (M or N), K, leading dimension
    (200, 256, None), (264, 64, None), (8, 32, None), (136, 96, 136), (520, 160, 528), (4104, 64, None),
    (1000, 512, 1008), (256, 256, None), (248, 32, 256), (392, 128, None),
]


@pytest.mark.parametrize("rows_tile", [128, 256])
@pytest.mark.parametrize("rows,K,ld", EDGE_SHAPES)
def test_row_contiguous_operand_stays_inside_with_the_clamp(rows_tile, rows, K, ld):
    ld = ld or rows
    assert max_overrun(False, rows_tile, rows, K, ld) <= 0


@pytest.mark.parametrize("rows_tile,fold", [(128, True), (256, True), (128, False), (256, False)])
@pytest.mark.parametrize("rows,K,ld", EDGE_SHAPES)
def test_k_contiguous_operand_stays_inside(rows_tile, fold, rows, K, ld):
    ld = ld or K
    ld = max(ld, K)
    assert max_overrun(True, rows_tile, rows, K, ld, fold=fold) <= 0


def test_without_the_clamp_an_edge_tile_reads_past_the_operand():
    # bf16 NN 256 x 200 x 256 on 128-wide tiles: B is 256 x 200, the second tile holds 72 valid columns
    over = max_overrun(False, 128, 200, 256, 200, clamp=False)
    assert over > 0 and over <= (128 - 8) * 2
    assert max_overrun(False, 128, 200, 256, 200, clamp=True) <= 0


def test_a_share_of_a_split_starts_at_a_later_slab():
    # the descriptor of a share starts at its first slab: the same bound holds from there
    for slab0 in (2, 4):
        assert max_overrun(False, 256, 328, 256, 328, slab0=slab0) <= 0
        assert max_overrun(True, 256, 328, 256, 256, slab0=slab0) <= 0
