// Host code of the library under AddressSanitizer and UndefinedBehaviorSanitizer (no GPU involved): the table
// solver, its exhaustive cross-check, the threshold, and the pass planner with an emulation of the addressing the
// kernels derive from its tables.  Built and run by tests/test_host_sanitizers.py.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "thc.h"
#include "thc_plan.hpp"

using namespace thc;

static uint64_t tile_base(const TileMap& m, uint32_t tile) {
  const uint32_t tib = tile & ((1u << m.nfixed) - 1u);
  uint32_t off = 0;
  for (int i = 0; i < 4; ++i) off |= ((tib >> m.fcum[i]) & m.fmask[i]) << m.fpos[i];
  return ((uint64_t)(tile >> m.nfixed) << m.L) | off;
}

static uint32_t tile_row(const TileMap& m, uint32_t r) {
  return ((r & ((1u << m.n0) - 1u)) << m.sh0) | ((r >> m.n0) << m.sh1);
}

// every coordinate of a span of 2^L is touched exactly once by the 2^(L-13) tiles of a strided pass
static int check_cover(const TileMap& m, bool first_pass_rows) {
  if (!m.L) return 1;
  const uint64_t span = 1ull << m.L;
  if (span > (1ull << 24)) return 0;                        // keep the run short; the Python test covers the rest
  std::vector<unsigned char> seen(span, 0);
  const uint32_t tiles = 1u << m.nfixed, W = 1u << m.logw;
  for (uint32_t t = 0; t < tiles; ++t) {
    const uint64_t base = tile_base(m, t);
    for (uint32_t idx = 0; idx < 8192; ++idx) {
      uint64_t o;
      if (first_pass_rows) o = (idx & 1023u) | ((uint64_t)(idx >> 10) << 13);
      else o = tile_row(m, idx >> m.logw) + (idx & (W - 1));
      const uint64_t j = base + o;
      if (j >= span || seen[j]) return 1;
      seen[j] = 1;
    }
  }
  return 0;
}

int main() {
  int bad = 0;
  for (int L = 10; L <= 27; ++L)
    for (uint32_t order = 0; order <= 1; ++order) {
      const Plan pl = make_plan(1ull << L, order);
      if (!pl.ok()) { std::printf("plan L=%d order=%u not ok\n", L, order); ++bad; continue; }
      int bits = pl.L1 + pl.R;
      for (int m = 0; m < pl.nmid; ++m) bits += pl.mid[m];
      if (bits != L) { std::printf("plan L=%d order=%u covers %d bits\n", L, order, bits); ++bad; }
      if (L >= 13) {
        if (pl.split) bad += check_cover(pl.lo, true);
        for (int m = 0; m < pl.nmid; ++m) bad += check_cover(pl.midmap[m], false);
        bad += check_cover(pl.hi, false);
        const TileMap lt = lo_tilemap(pl, 1ull << (L < 19 ? 19 : L));
        if (!pl.split) {
          // consecutive tiles in a permuted order: the bases are a permutation of the multiples of 8192
          const uint32_t tiles = 1u << lt.nfixed;
          std::vector<unsigned char> seen(tiles, 0);
          for (uint32_t t = 0; t < tiles; ++t) {
            const uint64_t b = tile_base(lt, t);
            if ((b & 8191u) || (b >> 13) >= tiles || seen[b >> 13]) { ++bad; break; }
            seen[b >> 13] = 1;
          }
        }
      }
    }
  uint8_t table[256];
  double cost = 0.0, cost2 = 0.0;
  uint64_t count = 0;
  for (uint32_t b = 1; b <= 4; ++b)
    for (uint32_t g = (1u << b) - 1; g <= (b == 4 ? 22u : 40u); g += 3) {
      if (thc_solve_table(b, g, 1.0 / 32, table, &cost) != THC_OK) ++bad;
      uint8_t t2[256];
      const int rc = thc_solve_table_bruteforce(b, g, 1.0 / 32, t2, &cost2, &count);
      if (rc == THC_OK) {
        for (uint32_t z = 0; z < (1u << b); ++z) bad += table[z] != t2[z];
      } else if (rc != THC_EUNSUPPORTED) {
        ++bad;
      }
    }
  if (thc_solve_table(8, 255, 1.0 / 1024, table, nullptr) != THC_OK) ++bad;
  if (thc_solve_table(4, 14, 0.1, table, nullptr) != THC_EINVAL) ++bad;       // g < 2^b - 1
  if (!(thc_threshold(1.0 / 32) > 2.15 && thc_threshold(1.0 / 32) < 2.16)) ++bad;
  std::printf("sanitizer run: %d problem(s)\n", bad);
  return bad ? 1 : 0;
}
