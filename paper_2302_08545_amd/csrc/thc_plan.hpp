// Host-side planner: how the butterfly stages of a block are split over the passes and how every pass tiles a
// block.  Plain C++ (no GPU types), so that it can be built and run under the host sanitizers.
#pragma once

#include <algorithm>
#include <cstdint>
#include <vector>

#include "thc.h"
#include "thc_tilemap.hpp"

namespace thc {

inline int ilog2(uint64_t v) {
  int l = 0;
  while ((1ull << l) < v) ++l;
  return l;
}

// Split of the log2(B) butterfly stages over the passes, and each pass's tiling (see TileMap).
//
// Stage order.  THC_ORDER_ASCENDING: bits 0, 1, ..., L-1.  THC_ORDER_SPLIT (blocks of at least 2^16):
// bits 0..9, 13, 14, 15, then 10, 11, 12, 16, ..., L-1.  In the split order the first pass works on eight rows
// of 1024 consecutive coordinates (4 KB) that are 32 KB apart instead of 8192 consecutive ones, which lets a
// workgroup -- hence its XCD -- stay on one value of byte-address bits 12..14 for both its reads and writes.
struct Plan {
  int L, L1;        // lo pass does L1 = min(L, 13) bits
  bool split;       // stage order THC_ORDER_SPLIT in effect
  int nmid;
  int mid[3];       // bit counts of the in-place middle passes
  int R;            // the last pass does R bits
  int bits[4][16];  // the butterfly bits of every pass after the first, in processing order (mids, then the last)
  TileMap lo, midmap[3], hi;
  bool ok() const {
    if (!lo.L || !hi.L) return false;
    for (int m = 0; m < nmid; ++m) if (!midmap[m].L) return false;
    return true;
  }
};

inline TileMap make_tilemap(int L, int logw, const std::vector<int>& rows, const int (&pref)[3]) {
  TileMap m{};
  m.L = (uint32_t)L;
  m.logw = (uint32_t)logw;
  m.nrows = (uint32_t)rows.size();
  m.nfixed = (uint32_t)(L - LOG_TILE);
  // rows: at most two runs of consecutive bit positions
  size_t run = 0;
  while (run + 1 < rows.size() && rows[run + 1] == rows[run] + 1) ++run;
  m.n0 = (uint32_t)(rows.empty() ? 0 : run + 1);
  m.sh0 = (uint32_t)(rows.empty() ? 0 : rows[0]);
  m.sh1 = (uint32_t)(m.n0 < rows.size() ? rows[m.n0] : 0);
  bool taken[32] = {};
  for (int r : rows) taken[r] = true;
  std::vector<int> fixed;
  for (int b : pref)
    if (b >= logw && b < L && !taken[b]) { fixed.push_back(b); taken[b] = true; }
  for (int b = logw; b < L; ++b)
    if (!taken[b]) fixed.push_back(b);
  // cut into runs of consecutive positions (at most four with the orders and splits used here)
  int nrun = 0;
  uint32_t cum = 0;
  for (size_t i = 0; i < fixed.size();) {
    size_t j = i;
    while (j + 1 < fixed.size() && fixed[j + 1] == fixed[j] + 1) ++j;
    if (nrun == 4) { m.L = 0; return m; }   // cannot happen; L = 0 makes validation fail loudly
    const uint32_t len = (uint32_t)(j - i + 1);
    m.fcum[nrun] = cum;
    m.fmask[nrun] = (1u << len) - 1u;
    m.fpos[nrun] = (uint32_t)fixed[i];
    cum += len;
    ++nrun;
    i = j + 1;
  }
  return m;
}

inline std::vector<int> bit_range(int lo, int hi) {
  std::vector<int> v;
  for (int b = lo; b < hi; ++b) v.push_back(b);
  return v;
}

inline Plan make_plan(uint64_t block, uint32_t stage_order) {
  Plan pl{};
  pl.L = ilog2(block);
  pl.L1 = pl.L < LOG_TILE ? pl.L : LOG_TILE;
  pl.split = stage_order == THC_ORDER_SPLIT && pl.L >= 16;
  // Up to 9 bits left after the lo pass: one strided pass takes them all (8 and 9 bits mean rows of only 128 and
  // 64 bytes, still far cheaper than another trip through HBM).  More than that: ceil(rem / 7) strided passes of
  // nearly equal size (wider rows make longer contiguous segments); the last one, fused with the quantizer or
  // the final scaling, gets the smallest.  In the split order the first of them starts with bits 10, 11, 12: its
  // rows are 1024 coordinates wide at most, so it must own all three, which any share of at least 3 bits guarantees.
  const int rem = pl.L - pl.L1;
  const int npass = rem <= 9 ? 1 : (rem + 6) / 7;
  pl.nmid = npass - 1;
  pl.R = rem / npass;
  for (int m = 0, left = rem - pl.R; m < pl.nmid; ++m) {
    pl.mid[m] = (left + (pl.nmid - m) - 1) / (pl.nmid - m);
    left -= pl.mid[m];
  }
  const int Lg = pl.L < LOG_TILE ? LOG_TILE : pl.L;   // blocks below 8192: tiles are just 8192 consecutive coordinates
  // bits still to do after the lo pass, in processing order
  std::vector<int> todo;
  if (pl.split) {
    todo = {10, 11, 12};
    for (int b = 16; b < pl.L; ++b) todo.push_back(b);
  } else {
    todo = bit_range(pl.L1, pl.L);
  }
  const int none[3] = {-1, -1, -1}, low[3] = {10, 11, 12}, grp[3] = {13, 14, 15};
  pl.lo = pl.split ? make_tilemap(Lg, 10, {13, 14, 15}, low) : make_tilemap(Lg, LOG_TILE, {}, none);
  size_t at = 0;
  for (int m = 0; m < pl.nmid; ++m) {
    std::vector<int> rows(todo.begin() + at, todo.begin() + at + pl.mid[m]);
    std::copy(rows.begin(), rows.end(), pl.bits[m]);
    pl.midmap[m] = make_tilemap(Lg, LOG_TILE - pl.mid[m], rows, pl.split ? grp : low);
    at += pl.mid[m];
  }
  std::vector<int> rows(todo.begin() + at, todo.end());
  std::copy(rows.begin(), rows.end(), pl.bits[pl.nmid]);
  pl.hi = make_tilemap(Lg, LOG_TILE - pl.R, rows, pl.split ? grp : low);
  return pl;
}

// Tiling of the first pass over `len` coordinates.  Consecutive 8192-coordinate tiles (ascending order, or blocks
// below 2^16) stream faster (measured: 5.7 against 5.3 TB/s) when the tile order is permuted inside spans of at least
// 2^19 coordinates so that the low three bits of the tile index, i.e. the XCD, select offset bits 16..18 rather
// than 13..15.  Vectors that are not whole spans keep the natural order.
inline TileMap lo_tilemap(const Plan& pl, uint64_t len) {
  if (pl.split) return pl.lo;
  const int span = pl.L < 19 ? 19 : pl.L;
  if (len & ((1ull << span) - 1)) return pl.lo;
  const int far[3] = {16, 17, 18};
  const TileMap m = make_tilemap(span, LOG_TILE, {}, far);
  return m.L ? m : pl.lo;
}

}  // namespace thc
