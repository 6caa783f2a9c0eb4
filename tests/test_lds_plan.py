"""Host-side check of the index arithmetic of the direct-to-LDS contraction kernel (csrc/lds_plan.h, compiled
here with g++): every LDS access stays inside the ring, the direct loads fill each operand tile exactly once,
and the transposed fragment reads hand every lane the matrix-core operand element it must hold.

The two hardware behaviours the arithmetic relies on are modelled as measured on gfx950:
  * a wave-wide 16-byte direct load puts lane L's bytes at destination + 16 L;
  * ds_read_b64_tr_b16: in each group of 16 lanes, lane i receives element (i % 4) of the 4 contiguous 16-bit
    values addressed by lanes (i / 4), (i / 4) + 4, (i / 4) + 8, (i / 4) + 12.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
STAGES, WAVES = 4, 8


@pytest.fixture(scope="module")
def plan(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("plan") / "plan_shim.so")
    subprocess.check_call(["g++", "-O1", "-shared", "-fPIC", "-o", so, os.path.join(HERE, "host_plan_shim.cpp")])
    lib = ctypes.CDLL(so)
    lib.plan_load_dst_bytes.restype = ctypes.c_uint
    return lib


def fill_stage(plan, stage):
    """What one k-tile's direct loads leave in LDS: element slot -> (operand, tile row, tile column)."""
    n = plan.plan_stage_elems()
    owner = -np.ones((STAGES * n, 3), dtype=np.int64)
    writes = np.zeros(STAGES * n, dtype=np.int64)
    for operand in range(2):
        for wave in range(WAVES):
            for q in range(2):
                base = plan.plan_load_dst_bytes(stage, operand, wave, q)
                assert base % 16 == 0
                for lane in range(64):
                    row = plan.plan_load_row(wave, lane) + 16 * q
                    chunk = plan.plan_load_chunk(wave, lane)
                    assert 0 <= row < plan.plan_tile_rows() and 0 <= chunk < plan.plan_row() // 8
                    e0 = (base + 16 * lane) // 2
                    for e in range(8):
                        owner[e0 + e] = (operand, row, 8 * chunk + e)
                        writes[e0 + e] += 1
    return owner, writes


@pytest.mark.parametrize("stage", range(STAGES))
def test_direct_loads_fill_each_stage_exactly_once_and_nothing_else(plan, stage):
    n = plan.plan_stage_elems()
    owner, writes = fill_stage(plan, stage)
    lo, hi = stage * n, (stage + 1) * n
    assert np.all(writes[lo:hi] == 1) and writes.sum() == n          # the stage, once; no byte outside it
    # every (operand, row, col) present once, and where kept_at() says
    seen = set()
    for operand in range(2):
        for row in range(plan.plan_tile_rows()):
            for col in range(plan.plan_row()):
                slot = lo + operand * plan.plan_operand_elems() + plan.plan_kept_at(row, col)
                assert tuple(owner[slot]) == (operand, row, col)
                seen.add(slot)
    assert len(seen) == n


def test_ring_fits_the_lds_allocation(plan):
    # 4 stages of 32 KB; the kernel asks for max(ring, epilogue staging) = 135232 bytes of LDS
    top = max(plan.plan_load_dst_bytes(STAGES - 1, 1, w, 1) + 1024 for w in range(WAVES))
    assert top == STAGES * plan.plan_stage_elems() * 2 == 131072 <= 135232


def test_fragment_reads_deliver_the_matrix_core_operand_layout(plan):
    """v_mfma_f32_32x32x16 wants, in lane l, operand[r = l % 32][k = 8 (l / 32) + 0..7] of the 32-wide block:
    k = tile row inside the 16-deep k-step, r = column inside the block.  Two transposed reads (rows f, f + 4)."""
    ROW = plan.plan_row()
    owner, _ = fill_stage(plan, 1)
    base = 1 * plan.plan_stage_elems()
    for operand in range(2):
        for block in range(8):
            for ks in range(2):
                addr = np.zeros((2, 64), dtype=np.int64)
                for half in range(2):
                    for lane in range(64):
                        a = plan.plan_frag_offset(lane, block) + ks * 16 * ROW + half * 4 * ROW
                        assert 0 <= a and a + 4 <= plan.plan_operand_elems()          # inside this operand's tile
                        assert (2 * a) % 8 == 0                                        # 8-byte aligned
                        addr[half, lane] = base + operand * plan.plan_operand_elems() + a
                for lane in range(64):
                    g, i = lane // 16, lane % 16
                    for half in range(2):
                        for j in range(4):
                            src_lane = 16 * g + (i // 4) + 4 * j
                            op, row, col = owner[addr[half, src_lane] + (i % 4)]
                            assert op == operand
                            assert row == 16 * ks + 8 * (lane // 32) + 4 * half + j
                            assert col == 32 * block + lane % 32


def test_transposed_reads_are_bank_conflict_free(plan):
    # a 64-bit LDS read is served 32 lanes at a time over 64 four-byte banks: the 32 lanes' 64 dwords must be
    # 64 different banks (this is what the swizzle is for: unpadded 512-byte rows would put rows t..t+3 on top
    # of each other)
    ROW = plan.plan_row()
    for block in range(8):
        for half_wave in range(2):
            banks = []
            for lane in range(32 * half_wave, 32 * half_wave + 32):
                byte = 2 * plan.plan_frag_offset(lane, block)
                banks += [(byte // 4) % 64, (byte // 4 + 1) % 64]
            assert len(set(banks)) == 64
