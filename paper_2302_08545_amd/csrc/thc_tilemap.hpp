// The tiling table shared by the host planner and the kernels (plain data, no GPU types).
#pragma once

#include <stdint.h>

namespace thc {

constexpr int LOG_TILE = 13;

// ---------------------------------------------------------------------------------------------
// Bit-permuted tiling.  Every transform pass cuts a block of 2^L coordinates into tiles of 8192: a tile is
// 2^nrows rows of 2^logw consecutive coordinates (nrows + logw = 13).  The offset bits of a coordinate
// inside its block are dealt out as
//   bits [0, logw)                          the column inside the row,
//   [sh0, sh0 + n0) and [sh1, ...)          the row index: its low n0 bits, then the rest,
//   runs (flen, fpos)                       the bit positions the tile index inside the block is scattered to.
// The host orders the runs so that the low three bits of the tile index (workgroup ids are dealt round-robin to
// the 8 XCDs) land on the offset bits that measured fastest for that pass.
// ---------------------------------------------------------------------------------------------
struct TileMap {
  // 32-bit fields throughout: the geometry is uniform per workgroup and stays in scalar registers
  uint32_t L;        // log2 of the span the tile index runs over (the block, or 13 for blocks below 8192)
  uint32_t logw;
  uint32_t nrows;
  uint32_t nfixed;   // = L - 13
  uint32_t n0, sh0, sh1;
  // the tile index inside the span, cut into up to four runs of consecutive bits: run i starts at bit fcum[i]
  // of the tile index, has mask fmask[i] = 2^length - 1 (0 for an unused run) and lands at offset bit fpos[i]
  uint32_t fcum[4];
  uint32_t fmask[4];
  uint32_t fpos[4];
};

}  // namespace thc
