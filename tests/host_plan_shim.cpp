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
