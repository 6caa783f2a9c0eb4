// Index arithmetic of the direct-to-LDS contraction kernel for tiles that are not 256 x 256
// (gemm_mfma_dma_shaped.hip.h), kept apart from the kernel so that a host compiler can check it.  Same hardware
// facts as lds_plan.h (a wave-wide 16-byte-per-lane direct load writes 1 KB of LDS, lane L's bytes at
// destination + 16 L; the lane pattern of ds_read_b64_tr_b16), generalised in two ways:
//   - an operand tile is 32 (t) rows of W elements, W a multiple of 64 (rows of 128 k bytes), kept as one flat
//     run of 16-byte chunks; 1 KB load n of an operand fills flat chunks 64 n .. 64 n + 63, which is not a whole
//     number of rows unless W is a multiple of 512, so every lane has its own (row, chunk) per load;
//   - the swizzle that keeps the transposed fragment reads (rows t .. t + 3 at one 64-byte column window) off
//     each other's banks depends on the row pitch: for pitches of 256 k bytes the four rows start on the same
//     bank and the 32-column block index is XORed with (t & 3) as in lds_plan.h; for pitches of 256 k + 128 bytes
//     rows t and t + 1 are already half the banks apart and the block index is XORed with ((t >> 1) & 1).
// Each operand's loads are dealt round-robin to the 8 waves: load n of the dY tile is instruction n / 8 of wave
// n % 8, the X tile's loads follow in the same way, so which operand an instruction loads does not depend on the
// wave.  Where an operand's load count is not a multiple of 8, the waves left without a load issue the instruction
// all the same, out of range (it fetches nothing and writes zeros to a spare 1 KB behind the ring), so that every
// wave has the same number of loads in flight and one wait count serves all.
#pragma once
#include <stdint.h>

#include "lds_plan.h"

namespace flashdp {
namespace shaped_plan {

constexpr int TILE_ROWS = 32;   // k-tile depth
constexpr int WAVES = 8;

constexpr FLASHDP_PLAN_HD int loads_of(int w) { return w / 16; }                                   // 1 KB loads per operand tile
constexpr FLASHDP_PLAN_HD int slots_of(int w) { return (loads_of(w) + WAVES - 1) / WAVES; }             // instructions per wave for it
constexpr FLASHDP_PLAN_HD int slots(int bm, int bn) { return slots_of(bm) + slots_of(bn); }           // per wave and k-tile
constexpr FLASHDP_PLAN_HD int stage_elems(int bm, int bn) { return TILE_ROWS * (bm + bn); }           // dY tile (bm wide), then X tile
constexpr FLASHDP_PLAN_HD uint32_t ring_bytes(int bm, int bn, int stages) { return (uint32_t)(stages * stage_elems(bm, bn)) * 2u; }
constexpr FLASHDP_PLAN_HD uint32_t lds_bytes_for_loads(int bm, int bn, int stages) { return ring_bytes(bm, bn, stages) + 1024u * WAVES; }

// instruction `slot` of every wave loads operand 0 (dY) or 1 (X) ...
constexpr FLASHDP_PLAN_HD int slot_operand(int bm, int bn, int slot) { return slot < slots_of(bm) ? 0 : 1; }
// ... namely this 1 KB of its tile, or nothing (-1)
FLASHDP_PLAN_HD int slot_index(int bm, int bn, int wave, int slot) {
  const int op = slot_operand(bm, bn, slot);
  const int n = WAVES * (op == 0 ? slot : slot - slots_of(bm)) + wave;
  return n < loads_of(op == 0 ? bm : bn) ? n : -1;
}
// LDS byte offset (from the start of the ring) the instruction writes its 1 KB to
FLASHDP_PLAN_HD uint32_t slot_dst_bytes(int bm, int bn, int stages, int stage, int wave, int slot) {
  const int n = slot_index(bm, bn, wave, slot);
  if (n < 0) return ring_bytes(bm, bn, stages) + 1024u * (uint32_t)wave;
  return (uint32_t)(stage * stage_elems(bm, bn) + slot_operand(bm, bn, slot) * TILE_ROWS * bm) * 2u + 1024u * (uint32_t)n;
}

// XOR applied to the 32-column block index of tile row `row` for an operand of width w
FLASHDP_PLAN_HD int swizzle(int row, int w) { return (w % 128 == 0) ? (row & 3) : ((row >> 1) & 1); }

// load n of an operand of width w: the tile row lane `lane` fills, and the 16-byte chunk of that row it fetches from
// memory (the chunk that belongs at the position the lane's bytes land on)
FLASHDP_PLAN_HD int lane_row(int w, int n, int lane) { return (64 * n + lane) / (w / 8); }
FLASHDP_PLAN_HD int lane_chunk(int w, int n, int lane) {
  const int pos = (64 * n + lane) % (w / 8);
  return pos ^ (swizzle(lane_row(w, n, lane), w) << 2);
}

// Where element (row, col) of an operand tile of width w is kept, in elements from the start of that tile.
FLASHDP_PLAN_HD int kept_at(int row, int col, int w) { return row * w + (((col >> 5) ^ swizzle(row, w)) << 5) + (col & 31); }

// Transposed fragment reads: lane addresses 4 contiguous elements at tile row lds_plan::frag_row (and + 4 for the
// second read; + 16 for the second k-step: all keep the swizzle of the row), columns 32 block + frag_col .. + 3.
FLASHDP_PLAN_HD int frag_offset(int lane, int block, int w) {
  return kept_at(lds_plan::frag_row(lane), 32 * block + lds_plan::frag_col(lane), w);
}

}  // namespace shaped_plan
}  // namespace flashdp
