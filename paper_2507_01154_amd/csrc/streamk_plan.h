// Who computes what in the balanced non-private gradient (gemm_mfma_streamk.hip.h), kept apart from the kernel so that
// a host compiler can check it: the walk of one XCD over its share of (block, k-tile) units, used unchanged by the
// kernel (every workgroup of the XCD) and by the host (to list the pieces of cut blocks for the second kernel).
#pragma once
#include <stdint.h>

#if defined(__HIPCC__)
#define FLASHDP_SK_HD __host__ __device__ __forceinline__
#else
#define FLASHDP_SK_HD static inline
#endif

namespace flashdp {

constexpr int STREAMK_XCDS = 8;            // ranges the work is cut into (workgroup id mod 8 = XCD)
constexpr int STREAMK_WG_PER_XCD = 32;     // one workgroup per tile of a block of 32 tiles
constexpr int STREAMK_SLOTS = 2 * STREAMK_XCDS;   // a range starts and ends with at most one cut block each
constexpr int STREAMK_MAX_CUT = 16;        // blocks that can be cut (each cut piece has its own slot)

// One piece of one range: block, k-range [k0, k1), and the partial slot it is stored to (-1: the whole reduction
// of the block lies in this piece, its tiles are stored straight to the output).
struct StreamKPiece { int block, k0, k1, slot; };

// Units are numbered block * nk_pad + k.  Range x is [x * units_per_xcd, (x + 1) * units_per_xcd), clipped to
// n_blocks * nk_pad; nk_pad and units_per_xcd are multiples of the ring depth, so every piece is.
// Calls f(piece) for every piece of range `xcd`, in order.
template <typename F>
FLASHDP_SK_HD void streamk_walk(int xcd, int n_blocks, int nk_pad, int units_per_xcd, F&& f) {
  const long total = (long)n_blocks * nk_pad;
  long u = (long)xcd * units_per_xcd;
  const long u_end = u + units_per_xcd < total ? u + units_per_xcd : total;
  int n_partial = 0;
  while (u < u_end) {
    StreamKPiece p;
    p.block = (int)(u / nk_pad);
    p.k0 = (int)(u - (long)p.block * nk_pad);
    const long left = u_end - u;
    p.k1 = p.k0 + left < nk_pad ? (int)(p.k0 + left) : nk_pad;
    const bool whole = p.k0 == 0 && p.k1 == nk_pad;
    p.slot = whole ? -1 : 2 * xcd + n_partial;
    if (!whole) ++n_partial;
    f(p);
    u += p.k1 - p.k0;
  }
}

// The host's choice of nk_pad and units_per_xcd for a problem: k-tiles of the batch-long reduction rounded up to the
// ring depth, and an eighth of all units rounded up likewise.
FLASHDP_SK_HD void streamk_sizes(long B, long T, long tiles, int bk, int stages, long* n_blocks, long* nk_pad, long* units_per_xcd) {
  *n_blocks = (tiles + STREAMK_WG_PER_XCD - 1) / STREAMK_WG_PER_XCD;
  const long nk = B * ((T + bk - 1) / bk);
  *nk_pad = (nk + stages - 1) / stages * stages;
  const long total = *n_blocks * *nk_pad;
  *units_per_xcd = ((total + STREAMK_XCDS - 1) / STREAMK_XCDS + stages - 1) / stages * stages;
}

}  // namespace flashdp
