// C-ABI of libthc (see include/thc.h): host-side validation and kernel dispatch.
#include "thc.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "thc_kernels.hpp"
#include "thc_plan.hpp"

namespace {

using namespace thc;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int validate(const thc_params* p) {
  if (!p) return THC_EINVAL;
  if (p->block < (1ull << 10) || p->block > (1ull << 27) || (p->block & (p->block - 1))) return THC_EINVAL;
  if (p->d == 0 || p->d % p->block || p->d >> 40) return THC_EINVAL;   // grids are 32-bit tile counts
  if (p->n < 1) return THC_EINVAL;
  if (p->n > THC_MAX_WORKERS) return THC_EUNSUPPORTED;
  if (p->b < 1 || p->b > 8) return THC_EINVAL;
  if (p->g < (1u << p->b) - 1 || p->g > 255) return THC_EINVAL;
  if (p->agg_bits < 1 || p->agg_bits > 16) return THC_EINVAL;
  if (p->in_dtype != THC_DTYPE_F32 && p->in_dtype != THC_DTYPE_BF16) return THC_EINVAL;
  if (!(p->t_p > 0.f) || !std::isfinite(p->t_p)) return THC_EINVAL;
  if (p->stage_order != THC_ORDER_ASCENDING && p->stage_order != THC_ORDER_SPLIT) return THC_EINVAL;
  if (p->group_log2 != 0 && (p->group_log2 < 10 || p->group_log2 > 40)) return THC_EINVAL;
  if (p->single_launch > 1) return THC_EINVAL;
  const uint32_t top = (1u << p->b) - 1;
  if (p->table[0] != 0 || p->table[top] != p->g) return THC_ETABLE;
  for (uint32_t z = 0; z < top; ++z)
    if (p->table[z] >= p->table[z + 1]) return THC_ETABLE;
  if ((uint64_t)p->g * p->n >= (1ull << p->agg_bits)) return THC_EOVERFLOW;
  return THC_OK;
}


// ---- workspace layout --------------------------------------------------------------------------------------
// [0, header)  status word of the last single-launch sweep (0 = fine), the rest reserved.  The header is 2 MiB
//              (4 KiB for small rings) so that the ring is aligned like the workspace itself: the passes' tilings
//              count on address bits up to 2^20.
// ring         the half-rotated vectors in flight: one group of blocks (launch-by-launch path) or a few block-sized
//              slots per vector (single-launch path); ring_floats(p, ef) binary32 values
// partials     n * (d >> min(L, 13)) binary64 partial sums of squares (one per 8192 coordinates, or per block)
// sync         counters of the single-launch path, K * SYNC_PER_UNIT words
// lut          device copy of the quantizer's grid-cell table, 256 words
//
// Launch-by-launch path: a group is a run of whole blocks of every vector in the call, sized so that the group's
// intermediate (all vectors of the call together) is about 2^group_log2 coordinates; the workspace does not grow
// with d.  Random streams are indexed by global coordinate, so the grouping never changes a result.
constexpr size_t WS_HEADER_BIG = 1u << 21, WS_HEADER_SMALL = 4096;
constexpr uint32_t DEFAULT_GROUP_LOG2 = 29;
constexpr uint32_t DEFAULT_GROUP_LOG2_SMALL = 25;   // with thc_params.single_launch: the caller is after a small workspace
// From a unit's last first-pass workgroup being dispatched to its range being visible, the chip gets through about
// this many workgroups (measured on the VGG16-shaped workload: trailing by fewer steps leaves consumers waiting,
// by more pushes the ring out of the memory-side cache).  A unit's next phase trails by at least that.
constexpr uint32_t LATENCY_WORKGROUPS = 1024;

uint64_t group_coords(const thc_params* p, uint32_t W) {
  const uint64_t target =
      1ull << (p->group_log2 ? p->group_log2 : p->single_launch ? DEFAULT_GROUP_LOG2_SMALL : DEFAULT_GROUP_LOG2);
  uint64_t gc = target / W / p->block * p->block;
  if (gc < p->block) gc = p->block;
  if (gc > p->d) gc = p->d;
  return gc;
}

// Shape of the single-launch sweep over W vectors (thc_pipeline.hpp), or ok = false where it does not apply:
// it is asked for by thc_params.single_launch and takes the split stage order, blocks of 2^17 .. 2^22 coordinates,
// at least four blocks, and the default grouping.
struct PipeShape {
  bool ok;
  uint32_t nphase, lag, slots;
};

PipeShape pipe_shape(const thc_params* p, const Plan& pl, uint32_t W, bool ef) {
  PipeShape sh{};
  const uint64_t K = p->d / p->block;
  sh.ok = p->single_launch == 1 && pl.split && pl.nmid == 0 && pl.L >= 17 && K >= 4 && K <= 65536 && p->group_log2 == 0;
  sh.nphase = ef ? 4 : 2;
  // A consumer should find its producers finished and published: they are `lag` steps ahead, a step being
  // nphase * Tu workgroups.
  const uint64_t per_step = (uint64_t)sh.nphase * ((uint64_t)W << pl.R);
  sh.lag = 1 + (uint32_t)((LATENCY_WORKGROUPS + per_step - 1) / per_step);
  sh.slots = (sh.nphase - 1) * sh.lag + 2;
  return sh;
}

uint64_t ring_floats(const thc_params* p, const Plan& pl, bool ef) {
  uint64_t need = group_coords(p, 1);
  const uint64_t all = (uint64_t)p->n * group_coords(p, p->n);
  if (all > need) need = all;
  for (uint32_t W : {1u, p->n}) {
    const PipeShape sh = pipe_shape(p, pl, W, ef);
    if (sh.ok && (uint64_t)sh.slots * W * p->block > need) need = (uint64_t)sh.slots * W * p->block;
  }
  return need;
}

size_t partial_count(const thc_params* p, const Plan& pl) { return (size_t)p->n * (size_t)(p->d >> pl.L1); }

size_t sync_words(const thc_params* p) {
  const uint64_t K = p->d / p->block;
  return (p->single_launch == 1 && K <= 65536) ? (size_t)K * SYNC_PER_UNIT : 0;
}

struct WsLayout {
  uint32_t* status;
  float* ring;
  double* partials;
  uint32_t* sync;
  uint32_t* lut;
  size_t bytes;
};

// The ring is sized for error feedback whenever the caller asked for it in thc_workspace_bytes; the calls take
// the layout that goes with what they are given (ef or not), which is the same or smaller.
WsLayout ws_layout(void* ws, const thc_params* p, const Plan& pl, bool ef) {
  char* base = static_cast<char*>(ws);
  WsLayout w{};
  const size_t ring_bytes = ring_floats(p, pl, ef) * sizeof(float);
  size_t at = ring_bytes >= WS_HEADER_BIG ? WS_HEADER_BIG : WS_HEADER_SMALL;
  w.status = reinterpret_cast<uint32_t*>(base);
  w.ring = reinterpret_cast<float*>(base + at);
  at += ring_bytes;
  w.partials = reinterpret_cast<double*>(base + at);
  at += partial_count(p, pl) * sizeof(double);
  w.sync = reinterpret_cast<uint32_t*>(base + at);
  at += sync_words(p) * sizeof(uint32_t);
  w.lut = reinterpret_cast<uint32_t*>(base + at);
  at += 256 * sizeof(uint32_t);
  w.bytes = at + 256;
  return w;
}

uint64_t tiles_of(uint64_t d) { return (d + TILE - 1) / TILE; }

// global coordinate of the buffers' first element
uint64_t base_coord(const thc_params* p) { return (uint64_t)p->first_block * p->block; }

void fill_lut(const thc_params* p, uint32_t (&lut)[256]) {
  const uint32_t top = (1u << p->b) - 1;
  for (uint32_t k = 0; k < 256; ++k) {
    const uint32_t kk = k < p->g ? k : p->g;
    uint32_t z0 = 0;
    while (z0 < top && p->table[z0 + 1] <= kk) ++z0;
    const uint32_t lo = p->table[z0];
    const uint32_t wd = z0 < top ? (uint32_t)(p->table[z0 + 1] - lo) : 255u;   // 255: the top value never rounds up
    lut[k] = lo | wd << 8 | z0 << 16;
  }
}

int check_launch() {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return THC_OK;
  std::fprintf(stderr, "libthc: kernel launch failed: %s\n", hipGetErrorString(e));
  return THC_ELAUNCH;
}

template <template <int> class Launcher, class... A>
void dispatch_0_7(int r, A&&... args) {
  switch (r) {
    case 0: Launcher<0>::run(args...); break;
    case 1: Launcher<1>::run(args...); break;
    case 2: Launcher<2>::run(args...); break;
    case 3: Launcher<3>::run(args...); break;
    case 4: Launcher<4>::run(args...); break;
    case 5: Launcher<5>::run(args...); break;
    case 6: Launcher<6>::run(args...); break;
    default: Launcher<7>::run(args...); break;
  }
}

// the last pass of a transform may take 8 or 9 bits
template <template <int> class Launcher, class... A>
void dispatch_0_9(int r, A&&... args) {
  switch (r) {
    case 8: Launcher<8>::run(args...); break;
    case 9: Launcher<9>::run(args...); break;
    default: dispatch_0_7<Launcher>(r, args...); break;
  }
}

// every launcher takes the number of vectors W of the launch: grid = (tiles, W)
template <int R> struct LaunchMid {
  static void run(const MidArgs& a, uint64_t tiles, uint32_t W, hipStream_t s) {
    k_mid<R><<<dim3((unsigned)tiles, W), dim3(NT), 0, s>>>(a);
  }
};
template <int R> struct LaunchQuant {
  static void run(const QuantArgs& a, bool cfold, uint64_t tiles, uint32_t W, hipStream_t s) {
    if (cfold && R >= 2) k_fwd_hi_quant<R, true><<<dim3((unsigned)tiles, W), dim3(NT), 0, s>>>(a);
    else k_fwd_hi_quant<R, false><<<dim3((unsigned)tiles, W), dim3(NT), 0, s>>>(a);
  }
};
template <int R> struct LaunchHiStore {
  static void run(const HiStoreArgs& a, uint64_t tiles, hipStream_t s) { k_fwd_hi_store<R><<<dim3((unsigned)tiles), dim3(NT), 0, s>>>(a); }
};
template <int R> struct LaunchInvHi {
  static void run(const InvHiArgs& a, uint64_t tiles, uint32_t W, hipStream_t s) {
    k_inv_hi<R><<<dim3((unsigned)tiles, W), dim3(NT), 0, s>>>(a);
  }
};

template <int L1, bool BF16, bool EF>
void launch_fwd_lo_k(const FwdLoArgs& a, bool split, bool norm_only, uint64_t tiles, uint32_t n, hipStream_t s) {
  const dim3 grid((unsigned)tiles, n);
  if constexpr (L1 == LOG_TILE) {
    if (split) {
      if (norm_only) k_fwd_lo<L1, BF16, EF, true, true><<<grid, dim3(NT), 0, s>>>(a);
      else k_fwd_lo<L1, BF16, EF, true, false><<<grid, dim3(NT), 0, s>>>(a);
      return;
    }
  }
  if (norm_only) k_fwd_lo<L1, BF16, EF, false, true><<<grid, dim3(NT), 0, s>>>(a);
  else k_fwd_lo<L1, BF16, EF, false, false><<<grid, dim3(NT), 0, s>>>(a);
}

template <int L1>
void launch_fwd_lo_t(const FwdLoArgs& a, bool bf16, bool ef, bool split, bool norm_only, uint64_t tiles, uint32_t n,
                     hipStream_t s) {
  if (bf16) {
    if (ef) launch_fwd_lo_k<L1, true, true>(a, split, norm_only, tiles, n, s);
    else launch_fwd_lo_k<L1, true, false>(a, split, norm_only, tiles, n, s);
  } else {
    if (ef) launch_fwd_lo_k<L1, false, true>(a, split, norm_only, tiles, n, s);
    else launch_fwd_lo_k<L1, false, false>(a, split, norm_only, tiles, n, s);
  }
}

void launch_fwd_lo(const Plan& pl, const FwdLoArgs& a, bool bf16, bool ef, bool norm_only, uint64_t tiles, uint32_t n,
                   hipStream_t s) {
  switch (pl.L1) {
    case 10: launch_fwd_lo_t<10>(a, bf16, ef, false, norm_only, tiles, n, s); break;
    case 11: launch_fwd_lo_t<11>(a, bf16, ef, false, norm_only, tiles, n, s); break;
    case 12: launch_fwd_lo_t<12>(a, bf16, ef, false, norm_only, tiles, n, s); break;
    default: launch_fwd_lo_t<13>(a, bf16, ef, pl.split, norm_only, tiles, n, s); break;
  }
}

void launch_range(const Plan& pl, const RangeArgs& r, hipStream_t s) {
  const uint64_t K = r.d >> pl.L;
  if (pl.L - pl.L1 <= 3) k_range_small<<<dim3((unsigned)((K + 255) / 256)), dim3(256), 0, s>>>(r);
  else k_range<<<dim3((unsigned)K), dim3(RANGE_NT), 0, s>>>(r);
}

void launch_inv_lo(const Plan& pl, const InvLoArgs& a, uint64_t tiles, uint32_t W, hipStream_t s) {
  const dim3 grid((unsigned)tiles, W), blk(NT);
  switch (pl.L1) {
    case 10: k_inv_lo<10, false><<<grid, blk, 0, s>>>(a); break;
    case 11: k_inv_lo<11, false><<<grid, blk, 0, s>>>(a); break;
    case 12: k_inv_lo<12, false><<<grid, blk, 0, s>>>(a); break;
    default:
      if (pl.split) k_inv_lo<13, true><<<grid, blk, 0, s>>>(a);
      else k_inv_lo<13, false><<<grid, blk, 0, s>>>(a);
      break;
  }
}

// middle passes of W vectors of `d` coordinates each, in place
void run_mids(const Plan& pl, float* x, uint64_t d, uint32_t W, hipStream_t s) {
  for (int m = 0; m < pl.nmid; ++m) {
    MidArgs a{x, d, pl.midmap[m]};
    dispatch_0_7<LaunchMid>(pl.mid[m], a, tiles_of(d), W, s);
  }
}

// inverse transform of W vectors of `len` coordinates that k_inv_lo is about to produce in `wsx`
void run_inverse(const thc_params* p, const Plan& pl, InvLoArgs lo, float* wsx, InvHiArgs hi, uint64_t len, uint32_t W,
                 hipStream_t s) {
  lo.tm = lo_tilemap(pl, len);
  lo.ws_x = wsx;
  lo.d = len;
  launch_inv_lo(pl, lo, tiles_of(len), W, s);
  run_mids(pl, wsx, len, W, s);
  hi.x = wsx;
  hi.d = len;
  hi.tm = pl.hi;
  hi.c = (float)(1.0 / std::sqrt((double)p->block));
  dispatch_0_9<LaunchInvHi>(pl.R, hi, tiles_of(len), W, s);
}

// Worker side of one round (Alg. 3) for W co-resident vectors, group by group:
//   first pass (x = grad + e, diagonal, 13 stages; with `range_out` also the norms) -> [range] -> middle passes ->
//   last pass + quantizer -> [error feedback: indices -> inverse first pass -> middle passes -> inverse last pass].
// Every kernel of a group covers all W vectors (grid.y), so a group costs the same number of launches for any W.
struct Forward {
  const thc_params* p;
  uint64_t round;
  uint32_t W;                  // vectors in the call
  uint32_t worker0;            // worker id of vector 0 (vector i is worker worker0 + i)
  const void* const* grads;    // W device pointers
  float* const* efs;           // W device pointers, or null: no error feedback
  float* range_out;            // not null: M_k from the W vectors' norms, written here and used
  const float* range_in;       // used when range_out is null
  uint8_t* const* packed;      // W device pointers
  void* ws;
  hipStream_t s;
};

template <int R>
void launch_pipe_forward(const PipeArgs& a, bool bf16, bool ef, unsigned grid, hipStream_t s) {
  if (bf16) {
    if (ef) k_pipe_forward<R, true, true><<<dim3(grid), dim3(NT), 0, s>>>(a);
    else k_pipe_forward<R, true, false><<<dim3(grid), dim3(NT), 0, s>>>(a);
  } else {
    if (ef) k_pipe_forward<R, false, true><<<dim3(grid), dim3(NT), 0, s>>>(a);
    else k_pipe_forward<R, false, false><<<dim3(grid), dim3(NT), 0, s>>>(a);
  }
}

// The whole sweep as one launch (plus a small one that clears the counters).
void run_forward_pipe(const Forward& f, const Plan& pl, const PipeShape& sh) {
  const thc_params* p = f.p;
  const bool bf16 = p->in_dtype == THC_DTYPE_BF16, ef = f.efs != nullptr;
  const WsLayout wl = ws_layout(f.ws, p, pl, ef);
  const uint32_t K = (uint32_t)(p->d / p->block);

  PipeSetupArgs su{};
  su.sync = wl.sync;
  su.nsync = (uint64_t)K * SYNC_PER_UNIT;
  su.status = wl.status;
  su.lut_out = wl.lut;
  fill_lut(p, su.lut);
  const unsigned setup_grid = (unsigned)((su.nsync + 4095) / 4096);
  k_pipe_setup<<<dim3(setup_grid ? setup_grid : 1), dim3(256), 0, f.s>>>(su);

  PipeArgs a{};
  for (uint32_t i = 0; i < f.W; ++i) {
    a.grads.p[i] = f.grads[i];
    if (ef) a.efs.p[i] = f.efs[i];
    a.packed.p[i] = f.packed[i];
  }
  a.ring = wl.ring;
  a.partials = wl.partials;
  a.pstride = p->d >> pl.L1;
  a.range_M = f.range_out ? f.range_out : const_cast<float*>(f.range_in);
  a.lut = wl.lut;
  a.sync = wl.sync;
  a.status = wl.status;
  a.d = p->d;
  a.j0 = base_coord(p);
  a.lo_tm = pl.lo;
  a.hi_tm = pl.hi;
  a.L = (uint32_t)pl.L;
  a.W = f.W;
  a.K = K;
  a.slots = sh.slots;
  a.lag = sh.lag;
  a.nphase = sh.nphase;
  a.compute_range = f.range_out ? 1u : 0u;
  a.b = p->b;
  a.g = p->g;
  a.round = (uint32_t)f.round;
  a.worker0 = f.worker0;
  a.k0 = (uint32_t)p->seed;
  a.k1 = (uint32_t)(p->seed >> 32);
  a.bf16 = bf16;
  a.c = (float)(1.0 / std::sqrt((double)p->block));
  a.t_p = p->t_p;
  std::memcpy(a.table, p->table, 256);
  const uint64_t Tu = (uint64_t)f.W << pl.R;
  const uint64_t steps = (uint64_t)K + (uint64_t)(sh.nphase - 1) * sh.lag;
  const uint64_t grid = steps * ((Tu >> 3) * sh.nphase + 1) * 8;
  switch (pl.R) {
    case 4: launch_pipe_forward<4>(a, bf16, ef, (unsigned)grid, f.s); break;
    case 5: launch_pipe_forward<5>(a, bf16, ef, (unsigned)grid, f.s); break;
    case 6: launch_pipe_forward<6>(a, bf16, ef, (unsigned)grid, f.s); break;
    case 7: launch_pipe_forward<7>(a, bf16, ef, (unsigned)grid, f.s); break;
    case 8: launch_pipe_forward<8>(a, bf16, ef, (unsigned)grid, f.s); break;
    default: launch_pipe_forward<9>(a, bf16, ef, (unsigned)grid, f.s); break;
  }
}

void run_forward(const Forward& f) {
  const thc_params* p = f.p;
  const Plan pl = make_plan(p->block, p->stage_order);
  {
    const PipeShape sh = pipe_shape(p, pl, f.W, f.efs != nullptr);
    const uint64_t Tu = (uint64_t)f.W << pl.R;
    const uint64_t grid = ((uint64_t)(p->d / p->block) + (uint64_t)(sh.nphase - 1) * sh.lag) * ((Tu >> 3) * sh.nphase + 1) * 8;
    if (sh.ok && grid < (1ull << 31)) {
      run_forward_pipe(f, pl, sh);
      return;
    }
  }
  const bool bf16 = p->in_dtype == THC_DTYPE_BF16;
  const size_t in_size = bf16 ? 2 : 4;
  const uint64_t gc = group_coords(p, f.W);
  const WsLayout wl = ws_layout(f.ws, p, pl, f.efs != nullptr);
  float* const slot = wl.ring;
  double* const partials = wl.partials;
  const float* const range = f.range_out ? f.range_out : f.range_in;

  QuantArgs q{};
  q.tm = pl.hi;
  q.L = (uint32_t)pl.L;
  q.b = p->b;
  q.g = p->g;
  q.round = (uint32_t)f.round;
  q.worker = f.worker0;
  q.k0 = (uint32_t)p->seed;
  q.k1 = (uint32_t)(p->seed >> 32);
  q.c = (float)(1.0 / std::sqrt((double)p->block));
  fill_lut(p, q.lut);   // per grid cell k: the largest index z0 with T[z0] <= k, its value and the gap to the next
  InvLoArgs ilo{};
  InvHiArgs ihi{};
  if (f.efs) {
    ilo.L = (uint32_t)pl.L;
    ilo.src_bits = p->b;
    ilo.use_table = 1;
    ilo.divisor = p->g;
    std::memcpy(ilo.table, p->table, 256);
    ihi.round = (uint32_t)f.round;
    ihi.k0 = q.k0;
    ihi.k1 = q.k1;
    ihi.mode = 1;
    ihi.bf16 = bf16;
  }
  for (uint64_t x0 = 0; x0 < p->d; x0 += gc) {
    const uint64_t len = p->d - x0 < gc ? p->d - x0 : gc;
    const uint64_t tiles = tiles_of(len);
    FwdLoArgs a{};
    for (uint32_t i = 0; i < f.W; ++i) {
      a.grads.p[i] = static_cast<const char*>(f.grads[i]) + x0 * in_size;
      if (f.efs) a.efs.p[i] = f.efs[i] + x0;
      q.packed.p[i] = f.packed[i] + x0 / 8 * p->b;
      if (f.efs) {
        ilo.src.p[i] = q.packed.p[i];
        ihi.out.p[i] = f.efs[i] + x0;
        ihi.grad.p[i] = a.grads.p[i];
      }
    }
    a.ws_x = slot;
    a.partials = f.range_out ? partials + (x0 >> pl.L1) : nullptr;
    a.pstride = p->d >> pl.L1;
    a.d = len;
    a.j0 = base_coord(p) + x0;
    a.round = (uint32_t)f.round;
    a.k0 = q.k0;
    a.k1 = q.k1;
    a.tm = lo_tilemap(pl, len);
    launch_fwd_lo(pl, a, bf16, f.efs != nullptr, false, tiles, f.W, f.s);
    if (f.range_out) {
      RangeArgs r{a.partials, f.range_out + x0 / p->block, a.pstride, len, f.W, (uint32_t)pl.L, (uint32_t)pl.L1, p->t_p};
      launch_range(pl, r, f.s);
    }
    run_mids(pl, slot, len, f.W, f.s);
    q.x = slot;
    q.range_M = range + x0 / p->block;
    q.d = len;
    q.j0 = a.j0;
    dispatch_0_9<LaunchQuant>(pl.R, q, (pl.L & 1) == 0, tiles, f.W, f.s);
    if (f.efs) {
      // e <- (grad + e) - RHT^-1(X_i): the group's slot is free again and takes the inverse's intermediate
      ilo.range_M = q.range_M;
      ihi.j0 = a.j0;
      run_inverse(p, pl, ilo, slot, ihi, len, f.W, f.s);
    }
  }
}

// ---- scratch of the entry point that allocates nothing -------------------------------------------------------
// One array per GPU the library's code object is loaded on, held until the process ends.  Its name is a host-side
// stand-in: the device address comes from hipGetSymbolAddress, once per device, with that device current.
constexpr uint64_t STATIC_SCRATCH_FLOATS = 1ull << 23;   // 32 MB
static __device__ __align__(256) float g_static_scratch[STATIC_SCRATCH_FLOATS];

constexpr int MAX_DEVICES = 64;
float* g_scratch_ptr[MAX_DEVICES] = {};

int static_scratch(float** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return THC_ELAUNCH;
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
    if (e != hipSuccess || !ptr) {
      std::fprintf(stderr, "libthc: hipGetSymbolAddress failed: %s\n", hipGetErrorString(e));
      return THC_ELAUNCH;
    }
    g_scratch_ptr[dev] = static_cast<float*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return THC_OK;
}

const char* const kNames[] = {"THC_OK", "THC_EINVAL", "THC_ETABLE", "THC_EOVERFLOW", "THC_EUNSUPPORTED", "THC_ELAUNCH"};

}  // namespace

extern "C" {

int thc_version(void) { return 200; }

const char* thc_strerror(int status) {
  const int i = -status;
  return (i >= 0 && i <= 5) ? kNames[i] : "THC_E?";
}

int thc_workspace_bytes(const thc_params* p, int ef_enabled, size_t* bytes_out) {
  const int rc = validate(p);
  if (rc) return rc;
  if (!bytes_out) return THC_EINVAL;
  const Plan pl = make_plan(p->block, p->stage_order);
  *bytes_out = ws_layout(nullptr, p, pl, ef_enabled != 0).bytes;
  return THC_OK;
}

int thc_describe_plan(const thc_params* p, uint32_t* out, size_t cap_records) {
  const int rc = validate(p);
  if (rc) return rc;
  const Plan pl = make_plan(p->block, p->stage_order);
  if (!pl.ok()) return THC_EUNSUPPORTED;
  const int npass = 2 + pl.nmid;
  if (!out) return npass;
  if (cap_records < (size_t)npass) return THC_EINVAL;
  auto put = [&](int rec, uint32_t kind, const int* bits, int nbits, const TileMap& m) {
    uint32_t* r = out + (size_t)rec * THC_PLAN_RECORD_WORDS;
    std::fill(r, r + THC_PLAN_RECORD_WORDS, 0xFFFFFFFFu);
    r[0] = kind;
    r[1] = (uint32_t)nbits;
    for (int i = 0; i < nbits; ++i) r[2 + i] = (uint32_t)bits[i];
    const uint32_t tm[19] = {m.L, m.logw, m.nrows, m.nfixed, m.n0, m.sh0, m.sh1, m.fcum[0], m.fcum[1], m.fcum[2],
                             m.fcum[3], m.fmask[0], m.fmask[1], m.fmask[2], m.fmask[3], m.fpos[0], m.fpos[1],
                             m.fpos[2], m.fpos[3]};
    std::copy(tm, tm + 19, r + 18);
  };
  int first[16];
  for (int i = 0; i < pl.L1; ++i) first[i] = (pl.split && i >= 10) ? i + 3 : i;
  put(0, pl.split ? 3u : 0u, first, pl.L1, lo_tilemap(pl, group_coords(p, p->n)));
  for (int m = 0; m < pl.nmid; ++m) put(1 + m, 1u, pl.bits[m], pl.mid[m], pl.midmap[m]);
  put(npass - 1, 2u, pl.bits[pl.nmid], pl.R, pl.hi);
  return npass;
}

namespace {

int check_vectors(const thc_params* p, const void* const* grads, const float* const* ef) {
  if (!grads) return THC_EINVAL;
  for (uint32_t i = 0; i < p->n; ++i) {
    if (!grads[i] || !aligned16(grads[i])) return THC_EINVAL;
    if (ef && (!ef[i] || !aligned16(ef[i]))) return THC_EINVAL;
  }
  return THC_OK;
}

}  // namespace

int thc_prepare_range(const thc_params* p, const void* const* grads, const float* const* ef, float* range_M, void* ws,
                      void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (!ws || !aligned16(ws) || !range_M || (reinterpret_cast<uintptr_t>(range_M) & 3u)) return THC_EINVAL;
  const int rv = check_vectors(p, grads, ef);
  if (rv) return rv;
  const Plan pl = make_plan(p->block, p->stage_order);
  hipStream_t s = static_cast<hipStream_t>(stream);
  // The same partial sums, in the same order, as the first pass of thc_compress_all takes them group by group: both
  // give the same M bit for bit.
  const bool bf16 = p->in_dtype == THC_DTYPE_BF16;
  double* const partials = ws_layout(ws, p, pl, false).partials;
  FwdLoArgs a{};
  for (uint32_t i = 0; i < p->n; ++i) {
    a.grads.p[i] = grads[i];
    if (ef) a.efs.p[i] = ef[i];
  }
  a.partials = partials;
  a.pstride = p->d >> pl.L1;
  a.d = p->d;
  a.tm = lo_tilemap(pl, p->d);
  launch_fwd_lo(pl, a, bf16, ef != nullptr, true, tiles_of(p->d), p->n, s);
  RangeArgs r{partials, range_M, p->d >> pl.L1, p->d, p->n, (uint32_t)pl.L, (uint32_t)pl.L1, p->t_p};
  launch_range(pl, r, s);
  return check_launch();
}

int thc_compress(const thc_params* p, uint32_t worker_id, uint64_t round, const void* grad, float* ef_inout,
                 const float* range_M, uint8_t* packed_out, void* ws, void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (worker_id >= p->n || round >> 32 || !range_M || !packed_out || !ws || !grad) return THC_EINVAL;
  if (!aligned16(packed_out) || !aligned16(ws) || !aligned16(grad)) return THC_EINVAL;
  if (ef_inout && !aligned16(ef_inout)) return THC_EINVAL;
  Forward f{p, round, 1, worker_id, &grad, ef_inout ? &ef_inout : nullptr, nullptr, range_M, &packed_out, ws,
            static_cast<hipStream_t>(stream)};
  run_forward(f);
  return check_launch();
}

int thc_compress_all(const thc_params* p, uint64_t round, const void* const* grads, float* const* ef_inout,
                     float* range_M, uint8_t* const* packed_out, void* ws, void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (round >> 32 || !ws || !aligned16(ws) || !range_M || (reinterpret_cast<uintptr_t>(range_M) & 3u) || !packed_out)
    return THC_EINVAL;
  const int rv = check_vectors(p, grads, ef_inout);
  if (rv) return rv;
  for (uint32_t i = 0; i < p->n; ++i)
    if (!packed_out[i] || !aligned16(packed_out[i])) return THC_EINVAL;
  Forward f{p, round, p->n, 0, grads, ef_inout, range_M, nullptr, packed_out, ws, static_cast<hipStream_t>(stream)};
  run_forward(f);
  return check_launch();
}

int thc_aggregate(const thc_params* p, const uint8_t* const* packed, void* agg_out, void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (!packed || !agg_out || !aligned16(agg_out)) return THC_EINVAL;
  for (uint32_t i = 0; i < p->n; ++i)
    if (!packed[i] || !aligned16(packed[i])) return THC_EINVAL;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (p->b == 4 && p->agg_bits == 8) {
    AggB4Args a{};
    for (uint32_t i = 0; i < p->n; ++i) a.packed.p[i] = packed[i];
    a.out = static_cast<uint8_t*>(agg_out);
    a.nvec = p->d / 32;
    a.n = p->n;
    std::memcpy(a.tb, p->table, 16);
    k_aggregate_b4w8<<<dim3((unsigned)((a.nvec + 255) / 256)), dim3(256), 0, s>>>(a);
  } else if (p->b == 2 && p->agg_bits == 8) {
    AggB2Args a{};
    for (uint32_t i = 0; i < p->n; ++i) a.packed.p[i] = packed[i];
    a.out = static_cast<uint8_t*>(agg_out);
    a.nvec = p->d / 64;
    a.n = p->n;
    std::memcpy(&a.tb, p->table, 4);
    k_aggregate_b2w8<<<dim3((unsigned)((a.nvec + 255) / 256)), dim3(256), 0, s>>>(a);
  } else if (p->b == 4) {
    AggB4W16Args a{};
    for (uint32_t i = 0; i < p->n; ++i) a.packed.p[i] = packed[i];
    a.out = static_cast<uint8_t*>(agg_out);
    a.nvec = p->d / 32;
    a.n = p->n;
    a.chunk = 255u / p->g;              // g <= 255, so at least one worker per run
    std::memcpy(a.tb, p->table, 16);
    const dim3 grid((unsigned)((a.nvec + 255) / 256)), blk(256);
    switch (p->agg_bits) {
      case 16: k_aggregate_b4w16<<<grid, blk, 0, s>>>(a); break;
#define THC_AGG_WX(W) case W: k_aggregate_b4wx<W><<<grid, blk, 0, s>>>(a); break;
      THC_AGG_WX(4) THC_AGG_WX(5) THC_AGG_WX(6) THC_AGG_WX(7) THC_AGG_WX(9) THC_AGG_WX(10) THC_AGG_WX(11)
      THC_AGG_WX(12) THC_AGG_WX(13) THC_AGG_WX(14) THC_AGG_WX(15)
#undef THC_AGG_WX
      default: return THC_EINVAL;       // 4-bit tables reach at least g = 15: the sums need 4 bits or more
    }
  } else {
    AggArgs a{};
    for (uint32_t i = 0; i < p->n; ++i) a.packed.p[i] = packed[i];
    a.out = agg_out;
    a.d = p->d;
    a.n = p->n;
    a.b = p->b;
    a.agg_bits = p->agg_bits;
    std::memcpy(a.table, p->table, 256);
    const uint64_t threads = p->d / 16;
    k_aggregate_generic<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s>>>(a);
  }
  return check_launch();
}

namespace {

// m + (Y/n)(M-m)/g and the inverse RHT, group by group through `slot` (room for `gc` coordinates, whole blocks)
void run_decompress(const thc_params* p, const Plan& pl, uint64_t round, const void* agg, const float* range_M,
                    float* out, float* slot, uint64_t gc, hipStream_t s) {
  InvLoArgs lo{};
  lo.L = (uint32_t)pl.L;
  lo.src_bits = p->agg_bits;
  lo.use_table = 0;
  lo.divisor = p->g * p->n;
  InvHiArgs hi{};
  hi.round = (uint32_t)round;
  hi.k0 = (uint32_t)p->seed;
  hi.k1 = (uint32_t)(p->seed >> 32);
  hi.mode = 0;
  for (uint64_t x0 = 0; x0 < p->d; x0 += gc) {
    const uint64_t len = p->d - x0 < gc ? p->d - x0 : gc;
    lo.src.p[0] = static_cast<const uint8_t*>(agg) + x0 / 8 * p->agg_bits;
    lo.range_M = range_M + x0 / p->block;
    hi.out.p[0] = out + x0;
    hi.j0 = base_coord(p) + x0;
    run_inverse(p, pl, lo, slot, hi, len, 1, s);
  }
}

}  // namespace

int thc_decompress(const thc_params* p, uint64_t round, const void* agg, const float* range_M, float* out,
                   void* ws, void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (round >> 32 || !agg || !range_M || !out || !ws) return THC_EINVAL;
  if (!aligned16(agg) || !aligned16(out) || !aligned16(ws)) return THC_EINVAL;
  const Plan pl = make_plan(p->block, p->stage_order);
  run_decompress(p, pl, round, agg, range_M, out, ws_layout(ws, p, pl, false).ring, group_coords(p, 1),
                 static_cast<hipStream_t>(stream));
  return check_launch();
}

int thc_decompress_noalloc(const thc_params* p, uint64_t round, const void* agg, const float* range_M, float* out,
                           void* stream) {
  const int rc = validate(p);
  if (rc) return rc;
  if (round >> 32 || !agg || !range_M || !out) return THC_EINVAL;
  if (!aligned16(agg) || !aligned16(out)) return THC_EINVAL;
  if (p->block > STATIC_SCRATCH_FLOATS) {
    std::fprintf(stderr, "libthc: thc_decompress_noalloc takes blocks of at most %llu coordinates (got %llu)\n",
                 (unsigned long long)STATIC_SCRATCH_FLOATS, (unsigned long long)p->block);
    return THC_EUNSUPPORTED;
  }
  float* scratch = nullptr;
  const int rs = static_scratch(&scratch);
  if (rs) return rs;
  const Plan pl = make_plan(p->block, p->stage_order);
  uint64_t gc = STATIC_SCRATCH_FLOATS / p->block * p->block;   // whole blocks that fit the scratch array
  if (gc > p->d) gc = p->d;
  run_decompress(p, pl, round, agg, range_M, out, scratch, gc, static_cast<hipStream_t>(stream));
  return check_launch();
}

// ---- uniform THC (Alg. 1) -----------------------------------------------------------------------

namespace {

int validate_uniform(const thc_params* p) {
  const int rc = validate(p);
  if (rc) return rc;
  if (p->g != (1u << p->b) - 1) return THC_ETABLE;     // identity table: T[z] = z (checked by validate: strictly increasing 0..g)
  return THC_OK;
}

// Workspace of the uniform entry points: with rotation the fully rotated vectors of all n workers (n*d binary32
// values, kept from thc_uniform_prepare_range to thc_uniform_compress), then per-tile minima and maxima.
size_t uni_x_bytes(const thc_params* p, int rotate) { return rotate ? (size_t)p->n * (size_t)p->d * sizeof(float) : 0; }

float* pmin_of(const thc_params* p, int rotate, void* ws) {
  return reinterpret_cast<float*>(static_cast<char*>(ws) + uni_x_bytes(p, rotate));
}

}  // namespace

int thc_uniform_workspace_bytes(const thc_params* p, int rotate, size_t* bytes_out) {
  const int rc = validate_uniform(p);
  if (rc) return rc;
  if (!bytes_out) return THC_EINVAL;
  const Plan pl = make_plan(p->block, p->stage_order);
  *bytes_out = uni_x_bytes(p, rotate) + partial_count(p, pl) * 2 * sizeof(float) + 256;
  return THC_OK;
}

int thc_uniform_prepare_range(const thc_params* p, uint64_t round, const void* const* grads, const float* const* ef,
                              int rotate, float* range_m, float* range_M, void* ws, void* stream) {
  const int rc = validate_uniform(p);
  if (rc) return rc;
  if (!grads || !ws || !aligned16(ws) || round >> 32 || !range_m || !range_M) return THC_EINVAL;
  for (uint32_t i = 0; i < p->n; ++i) {
    if (!grads[i] || !aligned16(grads[i])) return THC_EINVAL;
    if (ef && (!ef[i] || !aligned16(ef[i]))) return THC_EINVAL;
  }
  const Plan pl = make_plan(p->block, p->stage_order);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* pmin = pmin_of(p, rotate, ws);
  float* pmax = pmin + partial_count(p, pl);
  const size_t per_worker = (size_t)(p->d >> pl.L1);
  const bool bf16 = p->in_dtype == THC_DTYPE_BF16;
  if (rotate) {
    // full forward RHT of every worker, kept in the workspace
    FwdLoArgs a{};
    for (uint32_t i = 0; i < p->n; ++i) {
      a.grads.p[i] = grads[i];
      if (ef) a.efs.p[i] = ef[i];
    }
    a.ws_x = static_cast<float*>(ws);
    a.d = p->d;
    a.j0 = base_coord(p);
    a.round = (uint32_t)round;
    a.k0 = (uint32_t)p->seed;
    a.k1 = (uint32_t)(p->seed >> 32);
    a.tm = lo_tilemap(pl, p->d);
    launch_fwd_lo(pl, a, bf16, ef != nullptr, false, tiles_of(p->d), p->n, s);
    run_mids(pl, static_cast<float*>(ws), p->d, p->n, s);
    for (uint32_t i = 0; i < p->n; ++i) {
      float* wsx = static_cast<float*>(ws) + (size_t)i * p->d;
      HiStoreArgs h{wsx, pmin + i * per_worker, pmax + i * per_worker, p->d, pl.hi, (uint32_t)pl.L,
                    (float)(1.0 / std::sqrt((double)p->block))};
      dispatch_0_9<LaunchHiStore>(pl.R, h, tiles_of(p->d), s);
    }
  } else {
    MinMaxArgs a{};
    for (uint32_t i = 0; i < p->n; ++i) {
      a.grads.p[i] = grads[i];
      if (ef) a.efs.p[i] = ef[i];
    }
    a.pmin = pmin;
    a.pmax = pmax;
    a.d = p->d;
    a.L1 = (uint32_t)pl.L1;
    const dim3 grid((unsigned)tiles_of(p->d), p->n), blk(NT);
    if (bf16) { if (ef) k_minmax<true, true><<<grid, blk, 0, s>>>(a); else k_minmax<true, false><<<grid, blk, 0, s>>>(a); }
    else { if (ef) k_minmax<false, true><<<grid, blk, 0, s>>>(a); else k_minmax<false, false><<<grid, blk, 0, s>>>(a); }
  }
  MinMaxFinalArgs f{pmin, pmax, range_m, range_M, p->d, p->n, (uint32_t)pl.L, (uint32_t)pl.L1};
  k_minmax_final<<<dim3((unsigned)(p->d / p->block)), dim3(64), 0, s>>>(f);
  return check_launch();
}

int thc_uniform_compress(const thc_params* p, uint32_t worker_id, uint64_t round, const void* grad, float* ef_inout,
                         int rotate, const float* range_m, const float* range_M, uint8_t* packed_out, void* ws,
                         void* stream) {
  const int rc = validate_uniform(p);
  if (rc) return rc;
  if (worker_id >= p->n || round >> 32 || !range_m || !range_M || !packed_out || !aligned16(packed_out)) return THC_EINVAL;
  if (rotate && (!ws || !aligned16(ws))) return THC_EINVAL;
  if (!rotate && (!grad || !aligned16(grad))) return THC_EINVAL;
  if (ef_inout && (!grad || !aligned16(grad) || !aligned16(ef_inout))) return THC_EINVAL;
  const Plan pl = make_plan(p->block, p->stage_order);
  hipStream_t s = static_cast<hipStream_t>(stream);
  float* wsx = rotate ? static_cast<float*>(ws) + (size_t)worker_id * p->d : nullptr;
  UQuantArgs q{};
  q.x = wsx;
  q.grad = grad;
  q.ef = rotate ? nullptr : ef_inout;
  q.range_M = range_M;
  q.range_m = range_m;
  q.packed = packed_out;
  q.d = p->d;
  q.L = (uint32_t)pl.L;
  q.b = p->b;
  q.g = p->g;
  q.round = (uint32_t)round;
  q.worker = worker_id;
  q.k0 = (uint32_t)p->seed;
  q.k1 = (uint32_t)(p->seed >> 32);
  q.ef_update = (!rotate && ef_inout) ? 1u : 0u;
  q.j0 = base_coord(p);
  fill_lut(p, q.lut);
  const dim3 grid((unsigned)tiles_of(p->d)), blk(NT);
  if (p->in_dtype == THC_DTYPE_BF16) k_uniform_quant<true><<<grid, blk, 0, s>>>(q);
  else k_uniform_quant<false><<<grid, blk, 0, s>>>(q);
  if (rotate && ef_inout) {
    // e <- (grad + e) - RHT^-1(X_i): rebuild X_i from the indices, inverse transform, subtract
    InvLoArgs lo{};
    lo.src.p[0] = packed_out;
    lo.range_M = range_M;
    lo.range_m = range_m;
    lo.ws_x = wsx;
    lo.d = p->d;
    lo.L = (uint32_t)pl.L;
    lo.src_bits = p->b;
    lo.use_table = 1;
    lo.divisor = p->g;
    std::memcpy(lo.table, p->table, 256);
    InvHiArgs hi{};
    hi.out.p[0] = ef_inout;
    hi.grad.p[0] = grad;
    hi.round = (uint32_t)round;
    hi.k0 = q.k0;
    hi.k1 = q.k1;
    hi.mode = 1;
    hi.bf16 = p->in_dtype == THC_DTYPE_BF16;
    hi.j0 = base_coord(p);
    run_inverse(p, pl, lo, wsx, hi, p->d, 1, s);
  }
  return check_launch();
}

int thc_uniform_decompress(const thc_params* p, uint64_t round, const void* agg, int rotate, const float* range_m,
                           const float* range_M, float* out, void* ws, void* stream) {
  const int rc = validate_uniform(p);
  if (rc) return rc;
  if (round >> 32 || !agg || !range_m || !range_M || !out || !aligned16(agg) || !aligned16(out)) return THC_EINVAL;
  if (rotate && (!ws || !aligned16(ws))) return THC_EINVAL;
  const Plan pl = make_plan(p->block, p->stage_order);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (!rotate) {
    UDequantArgs a{agg, range_M, range_m, out, p->d, (uint32_t)pl.L, p->agg_bits, p->g * p->n};
    const uint64_t threads = p->d / 16;
    k_uniform_dequant<<<dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, s>>>(a);
    return check_launch();
  }
  float* wsx = static_cast<float*>(ws);
  InvLoArgs lo{};
  lo.src.p[0] = agg;
  lo.range_M = range_M;
  lo.range_m = range_m;
  lo.ws_x = wsx;
  lo.d = p->d;
  lo.L = (uint32_t)pl.L;
  lo.src_bits = p->agg_bits;
  lo.use_table = 0;
  lo.divisor = p->g * p->n;
  InvHiArgs hi{};
  hi.out.p[0] = out;
  hi.round = (uint32_t)round;
  hi.k0 = (uint32_t)p->seed;
  hi.k1 = (uint32_t)(p->seed >> 32);
  hi.mode = 0;
  hi.j0 = base_coord(p);
  run_inverse(p, pl, lo, wsx, hi, p->d, 1, s);
  return check_launch();
}

}  // extern "C"
