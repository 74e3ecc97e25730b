// Aggregation in the compressed domain (PS side of Alg. 2).
#pragma once

#include "thc_device.hpp"

namespace thc {

// ---------------------------------------------------------------------------------------------
// Aggregation (Alg. 2: Y = sum_i T[Z_i]; the PS only looks up and adds).  Generic path: one thread
// owns 16 consecutive coordinates of every stream; table in LDS.
// ---------------------------------------------------------------------------------------------
struct AggArgs {
  PtrArr packed;
  void* out;
  uint64_t d;
  uint32_t n, b, agg_bits;
  uint8_t table[256];
};

__global__ __launch_bounds__(256) void k_aggregate_generic(const AggArgs a) {
  __shared__ uint32_t tab[256];
  tab[threadIdx.x] = a.table[threadIdx.x];
  __syncthreads();
  const uint64_t j = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (j >= a.d) return;
  uint32_t acc[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0;
  for (uint32_t i = 0; i < a.n; ++i) {
    const uint8_t* s8 = static_cast<const uint8_t*>(a.packed.p[i]);
    if (a.b == 4) {
      const uint2 r = *reinterpret_cast<const uint2*>(s8 + (j >> 1));
      const uint32_t w[2] = {r.x, r.y};
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += tab[(w[e >> 3] >> (4 * (e & 7))) & 15u];
    } else if (a.b == 2) {
      const uint32_t w = *reinterpret_cast<const uint32_t*>(s8 + (j >> 2));
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += tab[(w >> (2 * e)) & 3u];
    } else if (a.b == 8) {
      const uint4 r = *reinterpret_cast<const uint4*>(s8 + j);
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += tab[(w[e >> 2] >> (8 * (e & 3))) & 255u];
    } else if (a.b == 1) {
      const uint32_t w = *reinterpret_cast<const uint16_t*>(s8 + (j >> 3));
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] += tab[(w >> e) & 1u];
    } else {
      uint32_t z0[8], z1[8];
      load_fields8(s8 + (j >> 3) * a.b, a.b, z0);
      load_fields8(s8 + ((j >> 3) + 1) * a.b, a.b, z1);
#pragma unroll
      for (int e = 0; e < 8; ++e) { acc[e] += tab[z0[e]]; acc[8 + e] += tab[z1[e]]; }
    }
  }
  uint8_t* out = static_cast<uint8_t*>(a.out);
  if (a.agg_bits == 8) {
    uint32_t w[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) w[k] = acc[4 * k] | acc[4 * k + 1] << 8 | acc[4 * k + 2] << 16 | acc[4 * k + 3] << 24;
    *reinterpret_cast<uint4*>(out + j) = make_uint4(w[0], w[1], w[2], w[3]);
  } else if (a.agg_bits == 16) {
    uint32_t w[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) w[k] = acc[2 * k] | acc[2 * k + 1] << 16;
    uint4* o = reinterpret_cast<uint4*>(out + 2 * j);
    o[0] = make_uint4(w[0], w[1], w[2], w[3]);
    o[1] = make_uint4(w[4], w[5], w[6], w[7]);
  } else {   // exact-width sums (Sec. 8.4: ceil(log2(g n + 1)) bits are enough)
    uint32_t z0[8], z1[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) { z0[e] = acc[e]; z1[e] = acc[8 + e]; }
    store_fields8(out + (j >> 3) * a.agg_bits, z0, a.agg_bits);
    store_fields8(out + ((j >> 3) + 1) * a.agg_bits, z1, a.agg_bits);
  }
}

// 4-bit indices -> 8-bit sums, the paper's prototype widths (Sec. 3).  One thread owns 32 coordinates
// (16 bytes of every stream); the 16-entry table sits in four registers and is applied to four
// nibbles at a time with byte permutes; sums of four coordinates share a register (no carry can
// cross a byte because g*n <= 255).
struct AggB4Args {
  PtrArr packed;
  uint8_t* out;
  uint64_t nvec;    // d / 32
  uint32_t n;
  uint32_t tb[4];   // table bytes 0..15, little endian
};

__device__ __forceinline__ uint32_t lut16x4(uint32_t sel, const uint32_t (&tb)[4]) {
  const uint32_t s7 = sel & 0x07070707u;
  const uint32_t lo = __builtin_amdgcn_perm(tb[1], tb[0], s7);
  const uint32_t hi = __builtin_amdgcn_perm(tb[3], tb[2], s7);
  const uint32_t m = ((sel & 0x08080808u) >> 3) * 0xFFu;
  return (hi & m) | (lo & ~m);
}

__global__ __launch_bounds__(256) void k_aggregate_b4w8(const AggB4Args a) {
  const uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= a.nvec) return;
  const uint32_t tb[4] = {a.tb[0], a.tb[1], a.tb[2], a.tb[3]};
  uint32_t ev[4] = {0, 0, 0, 0}, od[4] = {0, 0, 0, 0};
  for (uint32_t i = 0; i < a.n; ++i) {
    const uint4 r = reinterpret_cast<const uint4*>(a.packed.p[i])[v];
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      ev[k] += lut16x4(w[k] & 0x0F0F0F0Fu, tb);          // coordinates 8k + 0, 2, 4, 6
      od[k] += lut16x4((w[k] >> 4) & 0x0F0F0F0Fu, tb);   // coordinates 8k + 1, 3, 5, 7
    }
  }
  uint32_t o[8];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    o[2 * k] = __builtin_amdgcn_perm(od[k], ev[k], 0x05010400u);
    o[2 * k + 1] = __builtin_amdgcn_perm(od[k], ev[k], 0x07030602u);
  }
  uint4* dst = reinterpret_cast<uint4*>(a.out + v * 32);
  dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
  dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// 4-bit indices -> 16-bit sums (g*n above 255).  Same lookups; workers are taken in runs of `chunk` =
// floor(255 / g), inside which the byte-wise sums cannot carry, and every run is then widened into 16-bit lanes.
struct AggB4W16Args {
  PtrArr packed;
  uint8_t* out;
  uint64_t nvec;    // d / 32
  uint32_t n, chunk;
  uint32_t tb[4];
};

__global__ __launch_bounds__(256) void k_aggregate_b4w16(const AggB4W16Args a) {
  const uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= a.nvec) return;
  const uint32_t tb[4] = {a.tb[0], a.tb[1], a.tb[2], a.tb[3]};
  uint32_t acc[16];   // acc[4k + m] = sums of coordinates 8k + 2m (low half) and 8k + 2m + 1 (high half)
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0;
  for (uint32_t i0 = 0; i0 < a.n; i0 += a.chunk) {
    const uint32_t i1 = (i0 + a.chunk < a.n) ? i0 + a.chunk : a.n;
    uint32_t ev[4] = {0, 0, 0, 0}, od[4] = {0, 0, 0, 0};
    for (uint32_t i = i0; i < i1; ++i) {
      const uint4 r = reinterpret_cast<const uint4*>(a.packed.p[i])[v];
      const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        ev[k] += lut16x4(w[k] & 0x0F0F0F0Fu, tb);
        od[k] += lut16x4((w[k] >> 4) & 0x0F0F0F0Fu, tb);
      }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      acc[4 * k + 0] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C040C00u);
      acc[4 * k + 1] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C050C01u);
      acc[4 * k + 2] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C060C02u);
      acc[4 * k + 3] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C070C03u);
    }
  }
  uint4* dst = reinterpret_cast<uint4*>(a.out + v * 64);
#pragma unroll
  for (int k = 0; k < 4; ++k) dst[k] = make_uint4(acc[4 * k], acc[4 * k + 1], acc[4 * k + 2], acc[4 * k + 3]);
}

// 2-bit indices -> 8-bit sums.  One thread owns 64 coordinates (16 bytes of every stream); the four table
// values sit in one register; field f of every byte is looked up with one byte permute, so acc[k][f] holds the
// sums of coordinates 16k + 4*byte + f, and a 4x4 byte transpose restores coordinate order at the end.
struct AggB2Args {
  PtrArr packed;
  uint8_t* out;
  uint64_t nvec;    // d / 64
  uint32_t n;
  uint32_t tb;      // table bytes 0..3, little endian
};

__global__ __launch_bounds__(256) void k_aggregate_b2w8(const AggB2Args a) {
  const uint64_t v = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (v >= a.nvec) return;
  uint32_t acc[4][4];
#pragma unroll
  for (int k = 0; k < 4; ++k)
#pragma unroll
    for (int f = 0; f < 4; ++f) acc[k][f] = 0;
  for (uint32_t i = 0; i < a.n; ++i) {
    const uint4 r = reinterpret_cast<const uint4*>(a.packed.p[i])[v];
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int f = 0; f < 4; ++f) acc[k][f] += __builtin_amdgcn_perm(0u, a.tb, (w[k] >> (2 * f)) & 0x03030303u);
  }
  uint4* dst = reinterpret_cast<uint4*>(a.out + v * 64);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const uint32_t p0 = __builtin_amdgcn_perm(acc[k][1], acc[k][0], 0x05010400u);   // bytes 0, 1 of fields 0, 1
    const uint32_t p1 = __builtin_amdgcn_perm(acc[k][1], acc[k][0], 0x07030602u);   // bytes 2, 3
    const uint32_t q0 = __builtin_amdgcn_perm(acc[k][3], acc[k][2], 0x05010400u);
    const uint32_t q1 = __builtin_amdgcn_perm(acc[k][3], acc[k][2], 0x07030602u);
    dst[k] = make_uint4(__builtin_amdgcn_perm(q0, p0, 0x05040100u), __builtin_amdgcn_perm(q0, p0, 0x07060302u),
                        __builtin_amdgcn_perm(q1, p1, 0x05040100u), __builtin_amdgcn_perm(q1, p1, 0x07060302u));
  }
}

// 4-bit indices -> sums of any other width W (the exact width ceil(log2(g n + 1)) of Sec. 8.4, say).  Sums are
// formed as in k_aggregate_b4w16; a thread's 32 fields make exactly W dwords, which go through LDS so that the
// workgroup writes its 1024 * W bytes as consecutive 16-byte vectors.
template <int W>
__global__ __launch_bounds__(256) void k_aggregate_b4wx(const AggB4W16Args a) {
  __shared__ __align__(16) uint32_t stage[256 * W];
  const int t = threadIdx.x;
  const uint64_t v0 = (uint64_t)blockIdx.x * 256;
  const uint64_t v = v0 + t;
  if (v < a.nvec) {
    const uint32_t tb[4] = {a.tb[0], a.tb[1], a.tb[2], a.tb[3]};
    uint32_t acc[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0;
    for (uint32_t i0 = 0; i0 < a.n; i0 += a.chunk) {
      const uint32_t i1 = (i0 + a.chunk < a.n) ? i0 + a.chunk : a.n;
      uint32_t ev[4] = {0, 0, 0, 0}, od[4] = {0, 0, 0, 0};
      for (uint32_t i = i0; i < i1; ++i) {
        const uint4 r = reinterpret_cast<const uint4*>(a.packed.p[i])[v];
        const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          ev[k] += lut16x4(w[k] & 0x0F0F0F0Fu, tb);
          od[k] += lut16x4((w[k] >> 4) & 0x0F0F0F0Fu, tb);
        }
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        acc[4 * k + 0] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C040C00u);
        acc[4 * k + 1] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C050C01u);
        acc[4 * k + 2] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C060C02u);
        acc[4 * k + 3] += __builtin_amdgcn_perm(od[k], ev[k], 0x0C070C03u);
      }
    }
    // field e = coordinate e of the thread's 32: low or high half of acc[e / 2]; bits [e W, e W + W) of the output
    uint32_t out[W];
#pragma unroll
    for (int k = 0; k < W; ++k) out[k] = 0;
#pragma unroll
    for (int e = 0; e < 32; ++e) {
      const uint32_t f = (e & 1) ? acc[e >> 1] >> 16 : acc[e >> 1] & 0xFFFFu;
      const int pos = e * W, k = pos >> 5, sh = pos & 31;
      out[k] |= f << sh;
      if (sh + W > 32) out[k + 1] |= f >> (32 - sh);
    }
#pragma unroll
    for (int k = 0; k < W; ++k) stage[t * W + k] = out[k];
  }
  __syncthreads();
  const uint64_t left = a.nvec - v0;                       // threads of this workgroup that own coordinates
  const uint32_t nvec4 = (uint32_t)(left < 256 ? left : 256) * W / 4;   // a multiple of 8 W / 4: nvec is a multiple of 32
  uint4* dst = reinterpret_cast<uint4*>(a.out + v0 * 4 * W);
  const uint4* src = reinterpret_cast<const uint4*>(stage);
  for (uint32_t i = t; i < nvec4; i += 256) dst[i] = src[i];
}

}  // namespace thc
