// Host build of the index arithmetic of the direct-to-LDS contraction kernel (the same header the kernel
// includes), so that bounds and the swizzle can be checked on a machine without a GPU.  Not part of the product.
#include "../paper_2507_01154_amd/csrc/lds_plan.h"
using namespace flashdp::lds_plan;
extern "C" {
int plan_row() { return ROW; }
int plan_tile_rows() { return TILE_ROWS; }
int plan_stage_elems() { return STAGE_ELEMS; }
int plan_operand_elems() { return OPERAND_ELEMS; }
int plan_load_row(int wave, int lane) { return load_row(wave, lane); }
int plan_load_chunk(int wave, int lane) { return load_chunk(wave, lane); }
unsigned plan_load_dst_bytes(int stage, int operand, int wave, int q) { return load_dst_bytes(stage, operand, wave, q); }
int plan_kept_at(int row, int col) { return kept_at(row, col); }
int plan_frag_row(int lane) { return frag_row(lane); }
int plan_frag_col(int lane) { return frag_col(lane); }
int plan_frag_offset(int lane, int block) { return frag_offset(lane, block); }
}

// The walk of the balanced non-private gradient (which XCD computes which k-range of which block of tiles).
#include "../paper_2507_01154_amd/csrc/streamk_plan.h"
extern "C" {
void sk_sizes(long B, long T, long tiles, long* n_blocks, long* nk_pad, long* units) { flashdp::streamk_sizes(B, T, tiles, 32, 4, n_blocks, nk_pad, units); }
// writes up to cap pieces of range xcd as (block, k0, k1, slot) quadruples; returns the number of pieces
int sk_walk(int xcd, int n_blocks, int nk_pad, int units, int* out, int cap) {
  int n = 0;
  flashdp::streamk_walk(xcd, n_blocks, nk_pad, units, [&](const flashdp::StreamKPiece& p) {
    if (n < cap) { out[4 * n] = p.block; out[4 * n + 1] = p.k0; out[4 * n + 2] = p.k1; out[4 * n + 3] = p.slot; }
    ++n;
  });
  return n;
}
int sk_slots() { return flashdp::STREAMK_SLOTS; }
int sk_max_cut() { return flashdp::STREAMK_MAX_CUT; }
}

// Index arithmetic of the direct-to-LDS kernel for 384 x 192 and 192 x 384 tiles.
#include "../paper_2507_01154_amd/csrc/shaped_plan.h"
extern "C" {
int sp_slots(int bm, int bn) { return flashdp::shaped_plan::slots(bm, bn); }
int sp_stage_elems(int bm, int bn) { return flashdp::shaped_plan::stage_elems(bm, bn); }
unsigned sp_lds_bytes_for_loads(int bm, int bn, int stages) { return flashdp::shaped_plan::lds_bytes_for_loads(bm, bn, stages); }
int sp_slot_operand(int bm, int bn, int slot) { return flashdp::shaped_plan::slot_operand(bm, bn, slot); }
int sp_slot_index(int bm, int bn, int wave, int slot) { return flashdp::shaped_plan::slot_index(bm, bn, wave, slot); }
unsigned sp_slot_dst_bytes(int bm, int bn, int stages, int stage, int wave, int slot) { return flashdp::shaped_plan::slot_dst_bytes(bm, bn, stages, stage, wave, slot); }
int sp_lane_row(int w, int n, int lane) { return flashdp::shaped_plan::lane_row(w, n, lane); }
int sp_lane_chunk(int w, int n, int lane) { return flashdp::shaped_plan::lane_chunk(w, n, lane); }
int sp_kept_at(int row, int col, int w) { return flashdp::shaped_plan::kept_at(row, col, w); }
int sp_frag_offset(int lane, int block, int w) { return flashdp::shaped_plan::frag_offset(lane, block, w); }
}

// Index arithmetic of the direct-to-LDS kernel built on the 16x16x32 matrix-core instruction.
#include "../paper_2507_01154_amd/csrc/lds_plan16.h"
extern "C" {
int p16_load_row(int wave, int lane) { return flashdp::lds_plan16::load_row(wave, lane); }
int p16_load_chunk(int wave, int lane) { return flashdp::lds_plan16::load_chunk(wave, lane); }
unsigned p16_load_dst_bytes(int stage, int operand, int wave, int q) { return flashdp::lds_plan16::load_dst_bytes(stage, operand, wave, q); }
int p16_kept_at(int row, int col) { return flashdp::lds_plan16::kept_at(row, col); }
int p16_frag_offset(int lane, int block) { return flashdp::lds_plan16::frag_offset(lane, block); }
int p16_tile_base(int stage, int operand) { return flashdp::lds_plan16::tile_base(stage, operand); }
}
