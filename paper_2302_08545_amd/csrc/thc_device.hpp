// Device-side building blocks shared by the THC kernels (gfx950, wave64).
//
// Numeric contract: every butterfly is one binary32 add and one binary32 subtract, stages run in the order
// thc_params.stage_order fixes (the host hands each pass its bits as a TileMap), and nothing is contracted into a
// fused multiply-add unless written as __builtin_fmaf.  The file must be compiled with -ffp-contract=off.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "thc_tilemap.hpp"

namespace thc {

constexpr int TILE = 1 << LOG_TILE;   // coordinates one workgroup holds in LDS (32 KB of binary32)
constexpr int NT = 512;               // threads per workgroup: 16 coordinates each
constexpr int MAXW = 64;              // THC_MAX_WORKERS

struct PtrArr {
  const void* p[MAXW];
};

__device__ __forceinline__ uint64_t tm_base(const TileMap& m, uint32_t tile) {
  const uint32_t tib = tile & ((1u << m.nfixed) - 1u);
  uint32_t off = 0;
#pragma unroll
  for (int i = 0; i < 4; ++i) off |= ((tib >> m.fcum[i]) & m.fmask[i]) << m.fpos[i];
  return ((uint64_t)(tile >> m.nfixed) << m.L) | off;
}

// Kernels that walk a vector in consecutive 8192-coordinate tiles, one per workgroup: workgroup ids are dealt
// round-robin to the 8 XCDs, and streaming is faster (measured 5.7 against 5.3 TB/s) when an XCD keeps to its own
// value of byte-address bits 18..20 rather than 15..17.  Inside every whole group of 64 tiles the low three bits of
// the workgroup id therefore select tile bits 3..5.
__device__ __forceinline__ uint32_t xcd_tile(uint32_t wg, uint32_t ntiles) {
  return (wg | 63u) < ntiles ? (wg & ~63u) | ((wg & 7u) << 3) | ((wg >> 3) & 7u) : wg;
}

__device__ __forceinline__ uint32_t tm_row(const TileMap& m, uint32_t r) {
  return ((r & ((1u << m.n0) - 1u)) << m.sh0) | ((r >> m.n0) << m.sh1);
}

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One call yields 128 bits.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);   // three-input XOR in one instruction (truth table 0x96)
}

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c0;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
    const uint32_t n0 = xor3((uint32_t)(p1 >> 32), c1, k0);
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = xor3((uint32_t)(p0 >> 32), c3, k1);
    const uint32_t n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

constexpr uint32_t SIGN_STREAM = 0x80000000u;

// Word `(j >> 5) & 3` of the sign stream call that covers coordinate j (j a multiple of 32).
__device__ __forceinline__ uint32_t sign_word(uint64_t j, uint32_t round, uint32_t k0, uint32_t k1) {
  const uint64_t q = j >> 7;
  const uint4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), round, SIGN_STREAM, k0, k1);
  const uint32_t sel = (uint32_t)(j >> 5) & 3u;
  return sel == 0 ? r.x : sel == 1 ? r.y : sel == 2 ? r.z : r.w;
}

__device__ __forceinline__ float flip(float x, uint32_t bit /* 0 or 1 */) {
  return __uint_as_float(__float_as_uint(x) ^ (bit << 31));
}

// ---------------------------------------------------------------------------------------------
// In-register Walsh-Hadamard butterflies over 2^NB values, strides 1, 2, 4, ... in that order.
// ---------------------------------------------------------------------------------------------
template <int NB>
__device__ __forceinline__ void bfly(float (&v)[1 << NB]) {
#pragma unroll
  for (int s = 0; s < NB; ++s) {
    const int h = 1 << s;
#pragma unroll
    for (int j = 0; j < (1 << NB); ++j) {
      if ((j & h) == 0) {
        const float a = v[j], b = v[j + h];
        v[j] = a + b;
        v[j + h] = a - b;
      }
    }
  }
}

template <>
__device__ __forceinline__ void bfly<0>(float (&)[1]) {}

__device__ __forceinline__ void bfly_f4(float4& x) {   // strides 1 and 2 inside four consecutive values
  const float a = x.x + x.y, b = x.x - x.y, c = x.z + x.w, d = x.z - x.w;
  x.x = a + c; x.y = b + d; x.z = a - c; x.w = b - d;
}

// ---------------------------------------------------------------------------------------------
// LDS tile of TILE floats, three layouts (logical index -> physical slot):
//   PLAIN  identity.  Enough when every round reads 64 consecutive values per wave (P >= 6).
//   SWZ    bits 2..4 ^= bits 6..8: strided gathers of any round hit 32 distinct banks per half-wave.
//   PAD    four unused floats after every 64: the same property, and the 16 values a thread gathers in a
//          round sit at a constant physical stride, so their addresses are immediate offsets.
// All three keep four consecutive, 4-aligned values together as one 16-byte unit.
// ---------------------------------------------------------------------------------------------
enum Layout { PLAIN = 0, SWZ = 1, PAD = 2 };
constexpr int TILE_PAD = TILE + 4 * (TILE / 64);

__device__ __forceinline__ int swz(int i) { return i ^ (((i >> 6) & 7) << 2); }

template <Layout LY>
__device__ __forceinline__ int phys(int i) {
  if constexpr (LY == SWZ) return swz(i);
  else if constexpr (LY == PAD) return i + 4 * (i >> 6);
  else return i;
}

// One round: every thread gathers 16 values as (16 >> NB) groups of 2^NB values that differ in index
// bits [P, P+NB), runs the butterflies, and hands each result to sink(base, e << P, value): the value's
// tile index is base + (e << P), the two parts have no bits in common and the second is a constant.
template <int P, int NB, Layout LY, class Sink>
__device__ __forceinline__ void lds_round(const float* lds, int t, Sink&& sink) {
  constexpr int E = 1 << NB;
  constexpr int G = 16 >> NB;
  // physical distance between consecutive gathered values (PLAIN / PAD only)
  constexpr int ESTR = (LY == PAD && P >= 6) ? (1 << P) + 4 * ((1 << P) >> 6) : (1 << P);
  static_assert(LY != PAD || P >= 6 || P + NB <= 6, "a padded gather must not straddle a 64-value group");
#pragma unroll
  for (int gi = 0; gi < G; ++gi) {
    const int vt = t + NT * gi;
    const int base = (vt & ((1 << P) - 1)) | ((vt >> P) << (P + NB));
    const float* pb = lds + phys<LY>(base);
    float v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = (LY == SWZ) ? lds[swz(base + (e << P))] : pb[e * ESTR];
    bfly<NB>(v);
#pragma unroll
    for (int e = 0; e < E; ++e) sink(base, e << P, v[e]);
  }
}

// Stages for index bits [P, HI) on a tile resident in LDS.  When FUSE is set the last round hands its
// results to `sink` (typically a global store) instead of writing them back to LDS.
template <int P, int HI, bool FUSE, Layout LY, class Sink>
__device__ __forceinline__ void lds_stages(float* lds, int t, Sink&& sink) {
  constexpr int NB = (HI - P) < 4 ? (HI - P) : 4;
  constexpr bool LAST = (P + NB == HI);
  __syncthreads();
  if constexpr (LAST && FUSE) {
    lds_round<P, NB, LY>(lds, t, sink);
  } else {
    if constexpr (NB > 0) {
      lds_round<P, NB, LY>(lds, t, [&](int base, int eoff, float v) { lds[phys<LY>(base + eoff)] = v; });
    }
    if constexpr (!LAST) lds_stages<P + NB, HI, FUSE, LY>(lds, t, sink);
  }
}

__device__ __forceinline__ void bf4(float4& a, float4& b) {   // (a, b) -> (a + b, a - b), four columns at once
  const float4 s = make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w);
  b = make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w);
  a = s;
}

// fixed-order butterfly sum over the 64 lanes of a wave; every lane ends with the same total
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v += __shfl_xor(v, m, 64);
  return v;
}

// ---------------------------------------------------------------------------------------------
// Bit streams of w-bit fields (w <= 16), least-significant bits first: eight consecutive fields occupy
// exactly w consecutive bytes.  Generic (byte-wise) codec for the widths without a dedicated fast path.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void store_fields8(uint8_t* dst, const uint32_t (&z)[8], uint32_t w) {
  uint64_t lo = 0, hi = 0;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t pos = w * e;
    if (pos < 64) {
      lo |= (uint64_t)z[e] << pos;
      if (pos + w > 64) hi |= (uint64_t)z[e] >> (64 - pos);
    } else {
      hi |= (uint64_t)z[e] << (pos - 64);
    }
  }
  for (uint32_t i = 0; i < w; ++i) dst[i] = (uint8_t)(i < 8 ? lo >> (8 * i) : hi >> (8 * (i - 8)));
}

__device__ __forceinline__ void load_fields8(const uint8_t* src, uint32_t w, uint32_t (&z)[8]) {
  uint64_t lo = 0, hi = 0;
  for (uint32_t i = 0; i < w; ++i) {
    const uint64_t byte = src[i];
    if (i < 8) lo |= byte << (8 * i); else hi |= byte << (8 * (i - 8));
  }
  const uint32_t mask = (1u << w) - 1u;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const uint32_t pos = w * e;
    uint64_t v;
    if (pos < 64) {
      v = lo >> pos;
      if (pos + w > 64) v |= hi << (64 - pos);
    } else {
      v = hi >> (pos - 64);
    }
    z[e] = (uint32_t)v & mask;
  }
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }

}  // namespace thc
