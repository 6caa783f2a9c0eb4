// Index arithmetic of the direct-to-LDS contraction kernel, kept apart from the kernel so that a host
// compiler can check it: which element of an operand tile each lane fetches, where it lands in LDS, and
// which LDS addresses the transposed fragment reads use.  The hardware facts it encodes (measured on gfx950):
//   - one wave-wide 16-byte-per-lane direct load writes 1 KB of LDS, lane L's bytes at destination + 16 L;
//   - ds_read_b64_tr_b16: within 16 lanes, lane s supplies the address of 4 contiguous 16-bit values and lane i
//     receives element (i % 4) of lanes (i / 4), (i / 4) + 4, (i / 4) + 8, (i / 4) + 12.
// Operand tiles are 32 (t) x 256 elements of 16 bits (512-byte rows); the 16-byte chunk c of row t is kept at
// chunk position c ^ ((t & 3) << 2).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FLASHDP_PLAN_HD __host__ __device__ __forceinline__
#else
#define FLASHDP_PLAN_HD static inline
#endif

namespace flashdp {
namespace lds_plan {

constexpr int ROW = 256;              // elements per tile row
constexpr int TILE_ROWS = 32;         // k-tile depth
constexpr int OPERAND_ELEMS = TILE_ROWS * ROW;
constexpr int STAGE_ELEMS = 2 * OPERAND_ELEMS;   // dY tile, then X tile

// Direct loads: instruction q (0 or 1) of wave w (0..7) fills tile rows 16 q + 2 w and 16 q + 2 w + 1.
FLASHDP_PLAN_HD int load_row(int wave, int lane) { return 2 * wave + (lane >> 5); }   // add 16 q
// the chunk of that row the lane fetches, so that the row ends up swizzled in LDS
FLASHDP_PLAN_HD int load_chunk(int wave, int lane) { return (lane & 31) ^ ((load_row(wave, lane) & 3) << 2); }
// LDS byte offset (from the start of the ring) of the 1 KB instruction q of wave w writes; operand 0 = dY, 1 = X
FLASHDP_PLAN_HD uint32_t load_dst_bytes(int stage, int operand, int wave, int q) {
  return (uint32_t)(stage * STAGE_ELEMS + operand * OPERAND_ELEMS + (16 * q + 2 * wave) * ROW) * 2u;
}

// Where element (row, col) of an operand tile is kept, in elements from the start of that operand's tile.
FLASHDP_PLAN_HD int kept_at(int row, int col) { return row * ROW + (((col >> 5) ^ (row & 3)) << 5) + (col & 31); }

// Transposed fragment reads of one 16-deep k-step: the lane addresses 4 contiguous elements at tile row
// frag_row (and frag_row + 4 for the second read), columns 32 block + frag_col .. + 3.
FLASHDP_PLAN_HD int frag_row(int lane) { return 8 * (lane >> 5) + ((lane & 15) >> 2); }
FLASHDP_PLAN_HD int frag_col(int lane) { return 16 * ((lane >> 4) & 1) + 4 * (lane & 3); }
// element offset of the first read for 32-column block `block` (0..7); rows + 4 and + 16 keep row & 3
FLASHDP_PLAN_HD int frag_offset(int lane, int block) { return kept_at(frag_row(lane), 32 * block + frag_col(lane)); }

}  // namespace lds_plan
}  // namespace flashdp
