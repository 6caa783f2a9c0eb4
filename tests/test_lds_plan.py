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


# ---- the balanced non-private gradient: which XCD computes which k-range of which block (csrc/streamk_plan.h) ----

SK_SHAPES = [  # B, T, d_in, d_out
    (8, 2048, 5120, 5120), (8, 2048, 5120, 13824), (8, 2048, 13824, 5120), (4, 2048, 4096, 4096), (8, 1024, 768, 3072),
    (3, 160, 264, 392), (2, 100, 1544, 2056), (2, 192, 5120, 5120), (1, 33, 264, 24), (1, 1, 8, 8), (5, 31, 8192, 8192),
    (16, 4096, 256, 256), (2, 64, 16384, 16384),
]


@pytest.mark.parametrize("shape", SK_SHAPES)
def test_balanced_gradient_walk_covers_every_block_once(plan, shape):
    B, T, P, D = shape
    tiles = -(-D // 256) * -(-P // 256)
    nb, nkp, per = ctypes.c_long(), ctypes.c_long(), ctypes.c_long()
    plan.sk_sizes(B, T, tiles, ctypes.byref(nb), ctypes.byref(nkp), ctypes.byref(per))
    nb, nkp, per = nb.value, nkp.value, per.value
    assert nb == -(-tiles // 32) and nkp % 4 == 0 and nkp >= B * -(-T // 32) and per % 4 == 0 and 8 * per >= nb * nkp
    cover, cuts, slots = {}, {}, []
    buf = (ctypes.c_int * (4 * 64))()
    for x in range(8):
        n = plan.sk_walk(x, nb, nkp, per, buf, 64)
        assert n <= 64
        n_partial = 0
        for k in range(n):
            blk, k0, k1, slot = buf[4 * k], buf[4 * k + 1], buf[4 * k + 2], buf[4 * k + 3]
            assert 0 <= blk < nb and 0 <= k0 < k1 <= nkp and k0 % 4 == 0 and k1 % 4 == 0
            cover.setdefault(blk, []).append((k0, k1))
            if slot >= 0:
                assert slot == 2 * x + n_partial and slot < plan.sk_slots()     # at most two cut pieces per range
                n_partial += 1
                cuts.setdefault(blk, []).append(slot)
                slots.append(slot)
            else:
                assert (k0, k1) == (0, nkp)
    for blk in range(nb):                      # every block's reduction is covered exactly once, in order
        segs = cover[blk]
        assert segs[0][0] == 0 and segs[-1][1] == nkp and all(a[1] == b[0] for a, b in zip(segs, segs[1:]))
    assert len(set(slots)) == len(slots) and len(cuts) <= plan.sk_max_cut()
    assert all(2 <= len(v) <= 8 for v in cuts.values())       # a cut block has 2..8 pieces, one per range it spans
    # balance: no range has more than its share (a multiple of the ring depth) of units
    work = [sum(b[4 * k + 2] - b[4 * k + 1] for k in range(plan.sk_walk(x, nb, nkp, per, b, 64))) for x in range(8) for b in [buf]]
    assert max(work) <= per and sum(work) == nb * nkp


# ---- the same pipeline for 384 x 192 and 192 x 384 tiles (csrc/shaped_plan.h) ----

SHAPES = [(384, 192), (192, 384), (256, 256)]


def shaped_fill(plan, bm, bn, stage):
    """What one k-tile's direct loads leave in LDS: element slot -> (operand, tile row, tile column); loads that fetch
    nothing are recorded apart."""
    n = plan.sp_stage_elems(bm, bn)
    total = plan.sp_lds_bytes_for_loads(bm, bn, STAGES) // 2
    owner = -np.ones((total, 3), dtype=np.int64)
    writes = np.zeros(total, dtype=np.int64)
    idle = []
    for wave in range(WAVES):
        for slot in range(plan.sp_slots(bm, bn)):
            op = plan.sp_slot_operand(bm, bn, slot)
            k = plan.sp_slot_index(bm, bn, wave, slot)
            base = plan.sp_slot_dst_bytes(bm, bn, STAGES, stage, wave, slot)
            assert base % 1024 == 0 and base + 1024 <= 2 * total
            if k < 0:
                idle.append((wave, slot, base))
                continue
            w = bm if op == 0 else bn
            for lane in range(64):
                row, chunk = plan.sp_lane_row(w, k, lane), plan.sp_lane_chunk(w, k, lane)
                assert 0 <= row < 32 and 0 <= chunk < w // 8
                e0 = (base + 16 * lane) // 2
                for e in range(8):
                    owner[e0 + e] = (op, row, 8 * chunk + e)
                    writes[e0 + e] += 1
    return owner, writes, idle, n


@pytest.mark.parametrize("shape", SHAPES)
@pytest.mark.parametrize("stage", range(STAGES))
def test_shaped_loads_fill_each_stage_exactly_once(plan, shape, stage):
    bm, bn = shape
    owner, writes, idle, n = shaped_fill(plan, bm, bn, stage)
    lo, hi = stage * n, (stage + 1) * n
    assert np.all(writes[lo:hi] == 1) and writes.sum() == n
    for op, w in ((0, bm), (1, bn)):
        for row in range(32):
            for col in range(w):
                slot = lo + op * 32 * bm + plan.sp_kept_at(row, col, w)
                assert tuple(owner[slot]) == (op, row, col)
    # instructions without a load write (zeros) behind the ring, each wave to a 1 KB of its own, whatever the stage
    ring = STAGES * n * 2
    assert len(idle) == WAVES * plan.sp_slots(bm, bn) - (bm + bn) // 16
    assert all(base == ring + 1024 * wave for wave, _, base in idle)
    assert len({wave for wave, _, _ in idle}) == len(idle)          # at most one per wave: no two share a destination


@pytest.mark.parametrize("shape", SHAPES)
def test_shaped_fragment_reads_deliver_the_matrix_core_operand_layout(plan, shape):
    bm, bn = shape
    owner, _, _, n = shaped_fill(plan, bm, bn, 2)
    base = 2 * n
    for op, w in ((0, bm), (1, bn)):
        tile0 = base + op * 32 * bm
        for block in range(w // 32):
            for ks in range(2):
                addr = np.zeros((2, 64), dtype=np.int64)
                for half in range(2):
                    for lane in range(64):
                        a = plan.sp_frag_offset(lane, block, w) + ks * 16 * w + half * 4 * w
                        assert 0 <= a and a + 4 <= 32 * w and (2 * a) % 8 == 0
                        addr[half, lane] = tile0 + a
                for lane in range(64):
                    g, i = lane // 16, lane % 16
                    for half in range(2):
                        for j in range(4):
                            src_lane = 16 * g + (i // 4) + 4 * j
                            o, row, col = owner[addr[half, src_lane] + (i % 4)]
                            assert o == op
                            assert row == 16 * ks + 8 * (lane // 32) + 4 * half + j
                            assert col == 32 * block + lane % 32


@pytest.mark.parametrize("shape", SHAPES)
def test_shaped_transposed_reads_are_bank_conflict_free(plan, shape):
    bm, bn = shape
    for w, tile0 in ((bm, 0), (bn, 32 * bm)):
        for block in range(w // 32):
            for ks in range(2):
                for half in range(2):
                    for half_wave in range(2):
                        banks = []
                        for lane in range(32 * half_wave, 32 * half_wave + 32):
                            byte = 2 * (tile0 + plan.sp_frag_offset(lane, block, w) + ks * 16 * w + half * 4 * w)
                            banks += [(byte // 4) % 64, (byte // 4 + 1) % 64]
                        assert len(set(banks)) == 64


def test_shaped_plan_of_the_square_tile_is_the_square_plan(plan):
    for row in range(32):
        for col in range(256):
            assert plan.sp_kept_at(row, col, 256) == plan.plan_kept_at(row, col)
    for lane in range(64):
        for block in range(8):
            assert plan.sp_frag_offset(lane, block, 256) == plan.plan_frag_offset(lane, block)


# ---- the 256 x 256 kernel on the 16x16x32 matrix-core instruction (csrc/lds_plan16.h) ----

def fill_stage16(plan, stage):
    n = plan.plan_stage_elems()
    owner = -np.ones((STAGES * n, 3), dtype=np.int64)
    writes = np.zeros(STAGES * n, dtype=np.int64)
    for operand in range(2):
        for wave in range(WAVES):
            for q in range(2):
                base = plan.p16_load_dst_bytes(stage, operand, wave, q)
                for lane in range(64):
                    row = plan.p16_load_row(wave, lane) + 16 * q
                    chunk = plan.p16_load_chunk(wave, lane)
                    assert 0 <= row < 32 and 0 <= chunk < 32
                    e0 = (base + 16 * lane) // 2
                    for e in range(8):
                        owner[e0 + e] = (operand, row, 8 * chunk + e)
                        writes[e0 + e] += 1
    return owner, writes


@pytest.mark.parametrize("stage", range(STAGES))
def test_16x16x32_plan_loads_fill_each_stage_exactly_once(plan, stage):
    n, op_n = plan.plan_stage_elems(), plan.plan_operand_elems()
    owner, writes = fill_stage16(plan, stage)
    mine = np.zeros(STAGES * n, dtype=bool)
    for operand in range(2):                      # the ring is operand-major: 4 dY tiles, then 4 X tiles
        b = plan.p16_tile_base(stage, operand)
        assert b == (operand * STAGES + stage) * op_n
        mine[b:b + op_n] = True
    assert np.all(writes[mine] == 1) and writes.sum() == n       # this stage's two tiles, once; nothing else
    for operand in range(2):
        for row in range(32):
            for col in range(256):
                slot = plan.p16_tile_base(stage, operand) + plan.p16_kept_at(row, col)
                assert tuple(owner[slot]) == (operand, row, col)
    # every fragment read reaches every stage through the 16-bit offset field: stage offset + second read + k... < 64 KB
    assert 2 * ((STAGES - 1) * op_n + 4 * plan.plan_row()) < 65536


def test_16x16x32_plan_fragment_reads_deliver_the_operand_layout(plan):
    """v_mfma_f32_16x16x32 wants, in lane l, operand[r = l % 16][k = 8 (l / 16) + 0..7] of the 16-wide block: k = tile
    row inside the 32-deep k-tile, r = column inside the block.  Two transposed reads (rows f, f + 4)."""
    ROW = plan.plan_row()
    owner, _ = fill_stage16(plan, 3)
    for operand in range(2):
        for block in range(16):
            addr = np.zeros((2, 64), dtype=np.int64)
            for half in range(2):
                for lane in range(64):
                    a = plan.p16_frag_offset(lane, block) + half * 4 * ROW
                    assert 0 <= a and a + 4 <= plan.plan_operand_elems() and (2 * a) % 8 == 0
                    addr[half, lane] = plan.p16_tile_base(3, operand) + a
            for lane in range(64):
                g, i = lane // 16, lane % 16
                for half in range(2):
                    for j in range(4):
                        src_lane = 16 * g + (i // 4) + 4 * j
                        op, row, col = owner[addr[half, src_lane] + (i % 4)]
                        assert op == operand
                        assert row == 8 * (lane // 16) + 4 * half + j
                        assert col == 16 * block + lane % 16


def test_16x16x32_plan_transposed_reads_are_bank_conflict_free(plan):
    ROW = plan.plan_row()
    for block in range(16):
        for half in range(2):
            for half_wave in range(2):
                banks = []
                for lane in range(32 * half_wave, 32 * half_wave + 32):
                    byte = 2 * (plan.p16_frag_offset(lane, block) + half * 4 * ROW)
                    banks += [(byte // 4) % 64, (byte // 4 + 1) % 64]
                assert len(set(banks)) == 64
