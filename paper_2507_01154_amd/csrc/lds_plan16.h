// Index arithmetic of the direct-to-LDS contraction kernel built on the 16x16x32 matrix-core instruction
// (gemm_mfma_dma16.hip.h), kept apart from the kernel so that a host compiler can check it.  Same tile (32 (t) rows
// of 256 elements per operand), same direct loads (instruction q of wave w fills tile rows 16 q + 2 w and + 1) as
// lds_plan.h; what differs is the fragment a lane needs and hence the swizzle:
//   - v_mfma_f32_16x16x32: lane l holds operand[r = l % 16][k = 8 (l / 16) + 0..7] of a 16-wide block, so the four
//     16-lane groups of a wave read tile rows 8 g + 0..3 (and + 4 with the second read) at one 32-byte column window;
//   - a 64-bit LDS read is served 32 lanes at a time: groups g and g + 1, i.e. tile rows t..t+3 and t+8..t+11, must
//     fall on eight different 32-byte bank windows.  The 16-byte chunk c of row t is therefore kept at position
//     c ^ (((t & 3) << 2) | (((t >> 3) & 1) << 1)): rows t..t+3 go to four different 64-byte windows as before, and
//     rows 8 further on to the other 32-byte half of each.
// The ring is laid out operand-major - the four stages' dY tiles (4 x 16 KB), then the four X tiles - so that a
// fragment read reaches any stage of its operand through the 16-bit offset field of the LDS instruction from one
// address register per fragment (stage-major, the 32 KB stage stride would need a register per fragment and stage).
#pragma once
#include <stdint.h>

#include "lds_plan.h"

namespace flashdp {
namespace lds_plan16 {

constexpr int ROW = lds_plan::ROW;
constexpr int TILE_ROWS = lds_plan::TILE_ROWS;
constexpr int OPERAND_ELEMS = lds_plan::OPERAND_ELEMS;
constexpr int STAGE_ELEMS = lds_plan::STAGE_ELEMS;
constexpr int STAGES = 4;

// element offset of operand `operand` (0 = dY, 1 = X) of stage `stage` from the start of the ring
FLASHDP_PLAN_HD int tile_base(int stage, int operand) { return (operand * STAGES + stage) * OPERAND_ELEMS; }

// XOR applied to the 16-byte chunk index of tile row t
FLASHDP_PLAN_HD int swizzle(int t) { return ((t & 3) << 2) | (((t >> 3) & 1) << 1); }

FLASHDP_PLAN_HD int load_row(int wave, int lane) { return lds_plan::load_row(wave, lane); }   // add 16 q
// the chunk of that row the lane fetches (rows + 16 have the same swizzle)
FLASHDP_PLAN_HD int load_chunk(int wave, int lane) { return (lane & 31) ^ swizzle(load_row(wave, lane)); }
FLASHDP_PLAN_HD uint32_t load_dst_bytes(int stage, int operand, int wave, int q) {
  return (uint32_t)(tile_base(stage, operand) + (16 * q + 2 * wave) * ROW) * 2u;
}

// Where element (row, col) of an operand tile is kept, in elements from the start of that operand's tile.
FLASHDP_PLAN_HD int kept_at(int row, int col) { return row * ROW + (((col >> 3) ^ swizzle(row)) << 3) + (col & 7); }

// Transposed fragment reads of one k-tile: the lane addresses 4 contiguous elements at tile row frag_row (and
// frag_row + 4 for the second read), columns 16 block + frag_col .. + 3.
FLASHDP_PLAN_HD int frag_row(int lane) { return 8 * (lane >> 4) + ((lane & 15) >> 2); }
FLASHDP_PLAN_HD int frag_col(int lane) { return 4 * (lane & 3); }
// element offset of the first read for 16-column block `block` (0..15); row + 4 keeps the swizzle of the row
FLASHDP_PLAN_HD int frag_offset(int lane, int block) { return kept_at(frag_row(lane), 16 * block + frag_col(lane)); }

}  // namespace lds_plan16
}  // namespace flashdp
