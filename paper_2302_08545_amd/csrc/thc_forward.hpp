// Forward transform passes, the range kernel and the quantizer (worker side of Alg. 3).
#pragma once

#include "thc_device.hpp"

namespace thc {

// ---------------------------------------------------------------------------------------------
// Forward "lo" pass (Alg. 3: x = grad + e; ||x||; first part of R = RHT(x) with the diagonal D^r).
// grid = (tiles, n workers).  Writes the half-rotated tile to ws_x[worker] and one partial sum of
// squares per min(B, 8192) coordinates.
// ---------------------------------------------------------------------------------------------
struct FwdLoArgs {
  PtrArr grads;
  PtrArr efs;          // unused without error feedback
  float* ws_x;         // n * d floats
  double* partials;    // per worker `pstride` doubles, one per min(B, 8192) coordinates; or null: no norms wanted
  uint64_t pstride;
  uint64_t d;
  uint64_t j0;         // global coordinate of the vectors' first element (a multiple of B): indexes the diagonal
  uint32_t round, k0, k1;
  TileMap tm;          // where the bits of the tile index land; the tile shape is a template parameter
};

// Tile index -> offset inside the tile's span for the "lo" passes.  XO = false: 8192 consecutive
// coordinates.  XO = true: eight rows of 1024 consecutive coordinates, rows at offset bits 13..15 (the
// workgroup's XCD then stays on one value of offset bits 10..12 for reads and writes alike).
template <bool XO>
__device__ __forceinline__ uint32_t lo_map(uint32_t idx) {
  return XO ? ((idx & 1023u) | ((idx >> 10) << 13)) : idx;
}

template <bool BF16>
__device__ __forceinline__ float4 load_grad4(const void* g, uint64_t j) {
  if constexpr (BF16) {
    const ushort4 h = *reinterpret_cast<const ushort4*>(static_cast<const uint16_t*>(g) + j);
    return make_float4(bf16_to_f32(h.x), bf16_to_f32(h.y), bf16_to_f32(h.z), bf16_to_f32(h.w));
  } else {
    return *reinterpret_cast<const float4*>(static_cast<const float*>(g) + j);
  }
}

struct alignas(16) SmemLo {
  float lds[TILE_PAD];
  uint32_t sgn[TILE / 32];
  double wsum[4][NT / 64];
};

// One tile of the pass: tile index `tile` of vector `worker`; `dst` is where coordinate 0 of that vector's
// half-rotated image lives (the tile's results go to dst[offset in the vector]).
template <int L1, bool BF16, bool EF, bool XO, bool NORM_ONLY, class A>
__device__ __forceinline__ void fwd_lo_tile(const A& a, uint32_t tile, uint32_t worker, float* dst_vec,
                                            SmemLo& sm) {
  static_assert(!XO || L1 == LOG_TILE, "the row-split tile needs blocks of at least 2^16");
  // Vectors are multiples of B, so only blocks shorter than a tile can leave the last tile partial.
  constexpr bool GUARD = L1 < LOG_TILE;
  float* const lds = sm.lds;
  uint32_t* const sgn = sm.sgn;
  double (*const wsum)[NT / 64] = sm.wsum;

  const int t = threadIdx.x;
  const void* grad = a.grads.p[worker];
  const float* ef = EF ? static_cast<const float*>(a.efs.p[worker]) : nullptr;
  const int wave = t >> 6, lane = t & 63;
  const uint64_t off = tm_base(a.tm, tile);   // coordinate of tile index 0

  // all loads of the tile are issued before anything waits on them
  float4 x[4], e[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint64_t j = off + lo_map<XO>(4u * (uint32_t)(i * NT + t));
    const bool ok = !GUARD || j < a.d;
    x[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    e[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (ok) {
      x[i] = load_grad4<BF16>(grad, j);
      if constexpr (EF) e[i] = *reinterpret_cast<const float4*>(ef + j);
    }
  }

  if (!NORM_ONLY && t < 64) {   // the tile's 8192 diagonal entries: 64 Philox calls of 128 bits
    const uint64_t q = (a.j0 + off + lo_map<XO>(128u * t)) >> 7;
    const uint4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), a.round, SIGN_STREAM, a.k0, a.k1);
    *reinterpret_cast<uint4*>(&sgn[4 * t]) = r;
  }
  if constexpr (EF) {
#pragma unroll
    for (int i = 0; i < 4; ++i) { x[i].x += e[i].x; x[i].y += e[i].y; x[i].z += e[i].z; x[i].w += e[i].w; }
  }
  // sum of squares in binary64 (a binary32 square is exact there)
  double acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const double p = (double)x[i].x, q = (double)x[i].y, r = (double)x[i].z, s = (double)x[i].w;
    acc[i] = __builtin_fma(s, s, __builtin_fma(r, r, __builtin_fma(q, q, p * p)));
  }
  // a thread's four float4 sit 2048 coordinates apart: they share a block only if the block is that large
  if constexpr (L1 >= 13) {
    const double s = wave_sum((acc[0] + acc[1]) + (acc[2] + acc[3]));
    if (lane == 0) wsum[0][wave] = s;
  } else if constexpr (L1 == 12) {
    const double s0 = wave_sum(acc[0] + acc[1]), s1 = wave_sum(acc[2] + acc[3]);
    if (lane == 0) { wsum[0][wave] = s0; wsum[1][wave] = s1; }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const double s = wave_sum(acc[i]);
      if (lane == 0) wsum[i][wave] = s;
    }
  }
  __syncthreads();   // diagonal bits and wave sums visible

  // partial sums: one per block of 2^L1 coordinates inside the tile, combined in a fixed order
  constexpr int NBLK = TILE >> L1;
  if (t < NBLK) {
    double s = 0.0;
    if constexpr (L1 >= 13) {
#pragma unroll
      for (int w = 0; w < 8; ++w) s += wsum[0][w];
    } else if constexpr (L1 == 12 || L1 == 11) {
#pragma unroll
      for (int w = 0; w < 8; ++w) s += wsum[t][w];
    } else {   // L1 == 10: block = 2 * i + (wave >> 2)
#pragma unroll
      for (int w = 0; w < 4; ++w) s += wsum[t >> 1][4 * (t & 1) + w];
    }
    // one partial per tile (all of it in one block) or, for blocks below 8192, per block of the linear tile
    // the row-split tile is not contiguous: its number stands in (the same block either way); a contiguous tile
    // is numbered by where it lies
    const uint64_t pidx = XO ? (uint64_t)tile : (off >> L1) + t;
    if (a.partials && pidx < (a.d >> L1)) a.partials[(uint64_t)worker * a.pstride + pidx] = s;
  }
  if constexpr (NORM_ONLY) return;

  // diagonal, strides 1 and 2, then into LDS
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int idx = 4 * (i * NT + t);
    const uint32_t bits = sgn[idx >> 5] >> (idx & 31);
    x[i].x = flip(x[i].x, bits & 1u);
    x[i].y = flip(x[i].y, (bits >> 1) & 1u);
    x[i].z = flip(x[i].z, (bits >> 2) & 1u);
    x[i].w = flip(x[i].w, (bits >> 3) & 1u);
    bfly_f4(x[i]);
    *reinterpret_cast<float4*>(&lds[phys<PAD>(idx)]) = x[i];
  }

  float* dst = dst_vec + off;
  const uint64_t left = a.d - off;   // coordinates of this tile that exist (tail tile of a short vector)
  lds_stages<2, L1, true, PAD>(lds, t, [&](int base, int eoff, float v) {
    if (!GUARD || (uint64_t)(base + eoff) < left) dst[lo_map<XO>(base) + lo_map<XO>(eoff)] = v;
  });
}

// One workgroup per tile (grid = (tiles, n workers)): measured on MI355X this streams faster than a
// persistent grid with software prefetch, the hardware dispatcher keeps four workgroups per CU in flight.
// NORM_ONLY: stop after the partial sums of squares (the norm exchange of Alg. 3 on its own): same sums, same order.
template <int L1, bool BF16, bool EF, bool XO, bool NORM_ONLY = false>
__global__ __launch_bounds__(NT) void k_fwd_lo(const FwdLoArgs a) {
  __shared__ SmemLo sm;
  fwd_lo_tile<L1, BF16, EF, XO, NORM_ONLY>(a, blockIdx.x, blockIdx.y, a.ws_x + (uint64_t)blockIdx.y * a.d, sm);
}

// ---------------------------------------------------------------------------------------------
// Range (Sec. 5.3; Alg. 3: M = (t_p / sqrt(d)) * max_i ||x_i||, per block).
// ---------------------------------------------------------------------------------------------
struct RangeArgs {
  const double* partials;   // per worker `pstride` doubles
  float* range_M;           // K
  uint64_t pstride;
  uint64_t d;
  uint32_t n, L, L1;
  float t_p;
};

constexpr int RANGE_NT = NT;

__device__ __forceinline__ float range_from_sum(double smax, float t_p, uint32_t L) {
  return (float)(((double)t_p * __builtin_sqrt(smax)) / __builtin_sqrt((double)(1ull << L)));
}

// Blocks of at most 8 tiles (up to 2^16 coordinates): one thread per block adds the block's partial sums of
// every worker in index order.
__global__ __launch_bounds__(256) void k_range_small(const RangeArgs a) {
  const uint64_t k = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (k >= (a.d >> a.L)) return;
  const uint32_t ppb = 1u << (a.L - a.L1);
  const uint64_t per_worker = a.pstride;
  double smax = 0.0;
  for (uint32_t i = 0; i < a.n; ++i) {
    const double* p = a.partials + (uint64_t)i * per_worker + k * ppb;
    double s = 0.0;
    for (uint32_t j = 0; j < ppb; ++j) s += p[j];
    smax = s > smax ? s : smax;
  }
  a.range_M[k] = range_from_sum(smax, a.t_p, a.L);
}

struct SmemRange {
  double wsum[MAXW][RANGE_NT / 64];
};

// Larger blocks: one workgroup of RANGE_NT threads per block k.  Sigma x^2 of every worker in a fixed summation
// order (thread-strided partial sums, wave butterflies, then the wave totals in sequence), the maximum over workers,
// and M, returned by thread 0 (other threads return 0).  `partials` points at this call's first partial sum.
__device__ __forceinline__ float block_range(const double* partials, uint64_t pstride, uint32_t n, uint32_t ppb,
                                             uint64_t k, float t_p, uint32_t L, SmemRange& sm) {
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  for (uint32_t i = 0; i < n; ++i) {
    const double* p = partials + (uint64_t)i * pstride + k * ppb;
    double s = 0.0;
    for (uint32_t j = t; j < ppb; j += RANGE_NT) s += p[j];
    s = wave_sum(s);
    if (lane == 0) sm.wsum[i][wave] = s;
  }
  __syncthreads();
  float M = 0.f;
  if (t == 0) {
    double smax = 0.0;
    for (uint32_t i = 0; i < n; ++i) {
      double s = 0.0;
      for (int w = 0; w < RANGE_NT / 64; ++w) s += sm.wsum[i][w];
      smax = s > smax ? s : smax;
    }
    M = range_from_sum(smax, t_p, L);
  }
  return M;
}

__global__ __launch_bounds__(RANGE_NT) void k_range(const RangeArgs a) {
  __shared__ SmemRange sm;
  const float M = block_range(a.partials, a.pstride, a.n, 1u << (a.L - a.L1), blockIdx.x, a.t_p, a.L, sm);
  if (threadIdx.x == 0) a.range_M[blockIdx.x] = M;
}

// ---------------------------------------------------------------------------------------------
// Shared addressing of the strided passes: a tile of 2^R rows by W = 8192 >> R columns (see TileMap).
// ---------------------------------------------------------------------------------------------
template <int R>
struct HiGeom {
  static constexpr int LOGW = LOG_TILE - R;
  static constexpr int W = 1 << LOGW;
  const TileMap& m;
  uint64_t base;   // coordinate of (row 0, col 0)
  __device__ HiGeom(uint32_t tile, const TileMap& m_) : m(m_), base(tm_base(m_, tile)) {}
  // offset of a tile index from `base`: 32 bits are enough (blocks are at most 2^27 coordinates), so device
  // addresses can be formed as uniform 64-bit base + 32-bit per-lane offset
  __device__ uint32_t off(int idx) const { return tm_row(m, (uint32_t)idx >> LOGW) + (uint32_t)(idx & (W - 1)); }
  __device__ uint64_t coord(int idx) const { return base + off(idx); }
};

// Front half of a strided pass with R >= 2 row bits (no bounds checks: such tiles are always whole).
// Each thread loads four rows (4 rho + 0..3) of four consecutive columns, finishes row bits 0 and 1 in
// registers, parks the tile in LDS (row-major, no padding) and runs row bits [2, 2 + NB1) through LDS: one
// round of up to four bits for R <= 7, which leaves NB2 = R - 2 - NB1 (0 or 1) top bits for the caller's
// epilogue; two rounds and nothing left for R = 8 and 9 (rows of 128 and 64 bytes: blocks of 2^21 and 2^22
// coordinates then need no pass in between).
template <int R>
struct HiSplit {
  static constexpr int LOGW = LOG_TILE - R;
  static constexpr int W = 1 << LOGW;
  static constexpr int NB1 = R > 7 ? R - 2 : ((R - 2) < 4 ? (R - 2) : 4);
  static constexpr int NB2 = R - 2 - NB1;
  static_assert(R >= 2 && R <= 9 && NB2 <= 1, "strided pass handles 2..9 row bits");
};

template <int R>
__device__ __forceinline__ void hi_issue_loads(const float* src, const HiGeom<R>& g, int t, float4 (&x)[4]) {
  using S = HiSplit<R>;
  const int cg = t & (S::W / 4 - 1), rho = t >> (S::LOGW - 2);
  const float* pb = src + g.base;
  const uint32_t o = tm_row(g.m, 4 * rho) + 4 * cg;
  const uint32_t p1 = tm_row(g.m, 1), p2 = tm_row(g.m, 2);   // rows 4 rho + {1, 2, 3}
  x[0] = *reinterpret_cast<const float4*>(pb + o);
  x[1] = *reinterpret_cast<const float4*>(pb + (o + p1));
  x[2] = *reinterpret_cast<const float4*>(pb + (o + p2));
  x[3] = *reinterpret_cast<const float4*>(pb + (o + p1 + p2));
}

// row bits 0 and 1 in registers, then the tile goes to LDS (row-major, no padding)
template <int R>
__device__ __forceinline__ void hi_r0_to_lds(float4 (&x)[4], float* lds, int t) {
  using S = HiSplit<R>;
  const int cg = t & (S::W / 4 - 1), rho = t >> (S::LOGW - 2);
  bf4(x[0], x[1]); bf4(x[2], x[3]);   // row bit 0
  bf4(x[0], x[2]); bf4(x[1], x[3]);   // row bit 1
  float* q = lds + (4 * rho) * S::W + 4 * cg;
  *reinterpret_cast<float4*>(q) = x[0];
  *reinterpret_cast<float4*>(q + S::W) = x[1];
  *reinterpret_cast<float4*>(q + 2 * S::W) = x[2];
  *reinterpret_cast<float4*>(q + 3 * S::W) = x[3];
}

// row bits [2, 2 + NB1)  <->  tile index bits [LOGW + 2, LOGW + 2 + NB1); ends with the tile readable
template <int R>
__device__ __forceinline__ void hi_round1(float* lds, int t) {
  using S = HiSplit<R>;
  lds_stages<S::LOGW + 2, S::LOGW + 2 + S::NB1, false, PLAIN>(lds, t, [](int, int, float) {});
  __syncthreads();
}

template <int R>
__device__ __forceinline__ void hi_front(const float* src, const HiGeom<R>& g, float* lds, int t) {
  float4 x[4];
  hi_issue_loads<R>(src, g, t, x);
  hi_r0_to_lds<R>(x, lds, t);
  hi_round1<R>(lds, t);
}

// Two groups of eight consecutive coordinates per thread, with the last row bit (if any) applied:
// tile index of each group in idx[], values in v[][].
template <int R>
__device__ __forceinline__ void hi_back_index(int t, int (&idx)[2]) {
  using S = HiSplit<R>;
  if constexpr (S::NB2 == 1) {
    const int oct = t & (S::W / 8 - 1), r = t >> (S::LOGW - 3);      // r < 2^(R-1)
    idx[0] = r * S::W + 8 * oct;
    idx[1] = idx[0] + (TILE >> 1);
  } else {
    idx[0] = 8 * t;
    idx[1] = 8 * (t + NT);
  }
}

template <int R>
__device__ __forceinline__ void hi_back(const float* lds, int t, int (&idx)[2], float (&v)[2][8]) {
  using S = HiSplit<R>;
  hi_back_index<R>(t, idx);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const float4 p0 = *reinterpret_cast<const float4*>(&lds[idx[h]]);
    const float4 p1 = *reinterpret_cast<const float4*>(&lds[idx[h] + 4]);
    v[h][0] = p0.x; v[h][1] = p0.y; v[h][2] = p0.z; v[h][3] = p0.w;
    v[h][4] = p1.x; v[h][5] = p1.y; v[h][6] = p1.z; v[h][7] = p1.w;
  }
  if constexpr (S::NB2 == 1) {
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const float a = v[0][e], b = v[1][e];
      v[0][e] = a + b;
      v[1][e] = a - b;
    }
  }
}

// generic (slow) front for R < 2 and partial tiles: whole transform part through LDS
template <int R>
__device__ __forceinline__ void hi_load_to_lds(const float* src, const HiGeom<R>& g, uint64_t d, float* lds, int t) {
  float4 v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint64_t j = g.coord(4 * (i * NT + t));
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j < d) v[i] = *reinterpret_cast<const float4*>(src + j);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) *reinterpret_cast<float4*>(&lds[4 * (i * NT + t)]) = v[i];
}

// ---------------------------------------------------------------------------------------------
// "mid" pass: R more bits, in place.
// ---------------------------------------------------------------------------------------------
struct MidArgs {
  float* x;   // d floats per worker of the launch (grid.y = worker): half-rotated vectors
  uint64_t d;
  TileMap tm;
};

template <int R>
__global__ __launch_bounds__(NT) void k_mid(MidArgs a) {
  __shared__ __align__(16) float lds[TILE];
  const int t = threadIdx.x;
  const HiGeom<R> g(blockIdx.x, a.tm);
  a.x += (uint64_t)blockIdx.y * a.d;
  if constexpr (R >= 2) {
    hi_front<R>(a.x, g, lds, t);
    int idx[2];
    float v[2][8];
    hi_back<R>(lds, t, idx, v);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float* o = a.x + g.coord(idx[h]);
      *reinterpret_cast<float4*>(o) = make_float4(v[h][0], v[h][1], v[h][2], v[h][3]);
      *reinterpret_cast<float4*>(o + 4) = make_float4(v[h][4], v[h][5], v[h][6], v[h][7]);
    }
  } else {
    hi_load_to_lds<R>(a.x, g, a.d, lds, t);
    lds_stages<LOG_TILE - R, LOG_TILE, false, PLAIN>(lds, t, [](int, int, float) {});
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = 4 * (i * NT + t);
      const uint64_t j = g.coord(idx);
      if (j < a.d) *reinterpret_cast<float4*>(a.x + j) = *reinterpret_cast<const float4*>(&lds[idx]);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Forward "hi" pass + main stage, worker side (Alg. 3: R = RHT(x) finished; clamp to [-M, M];
// stochastic quantization onto the table's values (Sec. 4.1); Z = T^-1[Y] (Alg. 2); bit-pack).
//
// Per coordinate, in binary32:  v = h * c;  x' = med(v, -M, M);  y16 = (x' + M) * (scale * 2^16);
// k = floor(y16 / 2^16);  (lo, wd, z0) = LUT[k];  t16 = y16 - lo * 2^16;
// up iff (half + 1/2) * wd < t16  (one fused multiply-add, then compare);  z = z0 + up.
// The top table entry carries wd = 255 so that it can never round up.  When 1/sqrt(B) is a power of
// two (even log2 B) the multiplication by c is folded into M and the scale: that only moves exponents,
// so every rounding stays where it was.
// ---------------------------------------------------------------------------------------------
struct QuantArgs {
  const float* x;          // half-rotated vectors, d floats per worker of the launch (grid.y = worker)
  const float* range_M;    // K floats
  const float* range_m;    // K floats, or null: m = -M
  PtrArr packed;           // per worker of the launch: d*b/8 bytes, written
  uint64_t d;
  uint64_t j0;             // global coordinate of x[0] (a multiple of B): the random streams are indexed globally
  TileMap tm;
  uint32_t L;              // log2 B
  uint32_t b, g;
  uint32_t round, worker, k0, k1;   // worker: id of the launch's first worker (selects the rounding stream)
  float c;                 // 1/sqrt(B)
  uint32_t lut[256];       // per grid cell k: lo | wd << 8 | z0 << 16
};

struct QuantScalars {
  float M, lo, sc16, c;  // range [lo, M]; for even log2 B they and sc16 are pre-scaled by c, and c is unused
};

// WIDE = false: the fast form, on the grid position scaled by 2^16 (sc16 = scale * 2^16, range optionally folded
// with 1/sqrt(B)).  WIDE = true: ranges so narrow that scale * 2^16 would overflow binary32: the operations exactly
// as listed above (sc16 then holds the plain scale, the range is not folded), and the comparison scales t instead.
// Both forms take the same decisions: multiplying by a power of two commutes with every rounding involved.
template <bool CFOLD, bool WIDE = false>
__device__ __forceinline__ void quantize8(const float (&hv)[8], const uint4 rnd, const QuantScalars s,
                                          const uint4* lut, uint32_t (&z)[8]) {
  const uint32_t rw[4] = {rnd.x, rnd.y, rnd.z, rnd.w};
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const float v = (CFOLD && !WIDE) ? hv[e] : hv[e] * s.c;
    const float xc = __builtin_amdgcn_fmed3f(v, s.lo, s.M);
    const float y16 = (xc - s.lo) * s.sc16;          // WIDE: the grid position y itself
    const uint32_t ki = (uint32_t)y16;
    const uint4 ent = lut[(WIDE ? ki : ki >> 16) & 255u];
    const float t16 = WIDE ? (y16 - __uint_as_float(ent.x) * 0x1p-16f) * 65536.0f : y16 - __uint_as_float(ent.x);
    const float hf = (float)((e & 1) ? (rw[e >> 1] >> 16) : (rw[e >> 1] & 0xFFFFu));
    const float prod = __builtin_fmaf(hf, __uint_as_float(ent.y), __uint_as_float(ent.z));
    z[e] = ent.w + (prod < t16 ? 1u : 0u);
  }
}

// eight B-bit fields, field 0 in the least significant bits
template <int B>
__device__ __forceinline__ uint32_t pack8(const uint32_t (&z)[8]) {
  uint32_t w = z[7];
#pragma unroll
  for (int e = 6; e >= 0; --e) w = (w << B) | z[e];
  return w;
}

__device__ __forceinline__ void store_packed8(uint8_t* packed, uint64_t j, uint32_t b, const uint32_t (&z)[8]) {
  if (b == 4) {
    *reinterpret_cast<uint32_t*>(packed + (j >> 1)) = pack8<4>(z);
  } else if (b == 2) {
    *reinterpret_cast<uint16_t*>(packed + (j >> 2)) = (uint16_t)pack8<2>(z);
  } else if (b == 8) {
    const uint32_t w0 = z[0] | z[1] << 8 | z[2] << 16 | z[3] << 24;
    const uint32_t w1 = z[4] | z[5] << 8 | z[6] << 16 | z[7] << 24;
    *reinterpret_cast<uint2*>(packed + j) = make_uint2(w0, w1);
  } else if (b == 1) {
    packed[j >> 3] = (uint8_t)pack8<1>(z);
  } else {
    store_fields8(packed + (j >> 3) * b, z, b);
  }
}

// LDS entry of grid cell k: {lo * 2^16, wd, wd / 2 (all binary32, exact), z0}
__device__ __forceinline__ uint4 quant_lut_entry(uint32_t ent) {
  const float wd = (float)((ent >> 8) & 255u);
  return make_uint4(__float_as_uint((float)(ent & 255u) * 65536.0f), __float_as_uint(wd), __float_as_uint(0.5f * wd),
                    ent >> 16);
}

template <class A>
__device__ __forceinline__ void build_quant_lut(const A& a, uint4* lut, int t) {
  if (t < 256) lut[t] = quant_lut_entry(a.lut[t]);
}

// scale = g / (M - m): the width in binary64, the quotient rounded once to binary32.  Where that is not a finite
// number (M = m, or a width so small that the quotient overflows binary32) the range is empty: scale 0, every index 0.
__device__ __forceinline__ float scale_of(float M, float m, uint32_t g) {
  const float sc = (float)((double)g / ((double)M - (double)m));
  return sc <= 3.4028234663852886e38f ? sc : 0.f;     // also false for NaN
}

// scale * 2^16 (and the fold with 1/sqrt(B)) stay finite below this
constexpr float WIDE_SCALE = 0x1p110f;

// Per-block constants of the quantizer: the fast form whenever scale * 2^16 is representable.
__device__ __forceinline__ QuantScalars quant_scalars(float M, float m, uint32_t g, float c, bool cfold, bool& wide) {
  const float sc = scale_of(M, m, g);
  wide = sc >= WIDE_SCALE;
  if (wide) return QuantScalars{M, m, sc, c};
  const float sc16 = sc * 65536.0f;
  if (cfold) return QuantScalars{M * (1.0f / c), m * (1.0f / c), sc16 * c, c};
  return QuantScalars{M, m, sc16, c};
}

__device__ __forceinline__ float lower_of(const float* range_m, uint64_t blk, float M) {
  return range_m ? range_m[blk] : -M;
}

struct alignas(16) SmemQuant {
  float lds[TILE];
  uint32_t lut[256][4];   // uint4 entries
  float sQ[8][4];         // QuantScalars
  int sWide[8];
};

// One tile of the pass: tile index `tile` of the launch's vector `wk`, whose half-rotated image starts at xw.
template <int R, bool CFOLD, class A>
__device__ __forceinline__ void hi_quant_tile(const A& a, uint32_t tile, uint32_t wk, const float* xw,
                                              SmemQuant& sm) {
  float* const lds = sm.lds;
  uint4* const lut = reinterpret_cast<uint4*>(sm.lut);
  QuantScalars* const sQ = reinterpret_cast<QuantScalars*>(sm.sQ);
  int* const sWide = sm.sWide;

  const int t = threadIdx.x;
  uint8_t* const packed = static_cast<uint8_t*>(const_cast<void*>(a.packed.p[wk]));
  const uint32_t stream = a.worker + wk;

  if constexpr (R >= 2) {
    const HiGeom<R> g(tile, a.tm);
    float4 x[4];
    hi_issue_loads<R>(xw, g, t, x);             // tile loads first: everything below overlaps their latency
    build_quant_lut(a, lut, t);
    if (t == 0) {                               // the whole tile lies in one block
      const uint64_t blk = g.base >> a.L;
      const float M = a.range_M[blk], m = lower_of(a.range_m, blk, M);
      bool wide;
      sQ[0] = quant_scalars(M, m, a.g, a.c, CFOLD, wide);
      sWide[0] = wide;
    }
    hi_r0_to_lds<R>(x, lds, t);
    hi_round1<R>(lds, t);
    int idx[2];
    float v[2][8];
    hi_back<R>(lds, t, idx, v);
    const QuantScalars s = sQ[0];
    const bool wide = sWide[0] != 0;            // uniform over the workgroup
    const uint64_t q0 = (a.j0 + g.base) >> 3;   // tiles start on multiples of 64 coordinates
    uint8_t* const pk0 = packed + (g.base >> 3) * a.b;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t o = g.off(idx[h]);
      const uint64_t q = q0 + (o >> 3);
      const uint4 rnd = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), a.round, stream, a.k0, a.k1);
      uint32_t z[8];
      if (!wide) quantize8<CFOLD>(v[h], rnd, s, lut, z);
      else quantize8<CFOLD, true>(v[h], rnd, s, lut, z);
      store_packed8(pk0, o, a.b, z);
    }
  } else {
    const HiGeom<R> g(tile, a.tm);
    build_quant_lut(a, lut, t);
    // per-block scalars; a tile spans more than one block only when B < 8192 (then R == 0)
    const int nblk = a.L < LOG_TILE ? (TILE >> a.L) : 1;
    if (t < nblk) {
      const uint64_t blk = (g.base >> a.L) + t;
      float M = 0.f, m = 0.f;
      if (blk < (a.d >> a.L)) { M = a.range_M[blk]; m = lower_of(a.range_m, blk, M); }
      bool wide;
      sQ[t] = quant_scalars(M, m, a.g, a.c, false, wide);
      sWide[t] = wide;
    }
    hi_load_to_lds<R>(xw, g, a.d, lds, t);
    lds_stages<LOG_TILE - R, LOG_TILE, false, PLAIN>(lds, t, [](int, int, float) {});
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int idx = 8 * (t + NT * h);
      const uint64_t j = g.coord(idx);
      if (j >= a.d) continue;
      const int bt = a.L < LOG_TILE ? (idx >> a.L) : 0;
      const QuantScalars s = sQ[bt];
      const float4 p0 = *reinterpret_cast<const float4*>(&lds[idx]);
      const float4 p1 = *reinterpret_cast<const float4*>(&lds[idx + 4]);
      const float hv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
      const uint64_t q = (a.j0 + j) >> 3;
      const uint4 rnd = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), a.round, stream, a.k0, a.k1);
      uint32_t z[8];
      if (!sWide[bt]) quantize8<false>(hv, rnd, s, lut, z);
      else quantize8<false, true>(hv, rnd, s, lut, z);
      store_packed8(packed, j, a.b, z);
    }
  }
}

template <int R, bool CFOLD>
__global__ __launch_bounds__(NT, 8) void k_fwd_hi_quant(const QuantArgs a) {
  __shared__ SmemQuant sm;
  hi_quant_tile<R, CFOLD>(a, blockIdx.x, blockIdx.y, a.x + (uint64_t)blockIdx.y * a.d, sm);
}

}  // namespace thc
