// Uniform THC (Alg. 1): min/max ranges and uniform stochastic quantization.
#pragma once

#include "thc_inverse.hpp"

namespace thc {

// ---------------------------------------------------------------------------------------------
// Uniform THC (Alg. 1).  Preliminary stage: every worker's minimum and maximum per block, then the
// global ones.  Main stage: uniform stochastic quantization = the same quantizer with the identity
// table, on the gradients themselves or (ablation of App. C) on their RHT.
// Partial minima / maxima: one per min(B, 8192) coordinates per worker, like the partial sums of squares.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v = __builtin_fminf(v, __shfl_xor(v, m, 64));
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int m = 1; m < 64; m <<= 1) v = __builtin_fmaxf(v, __shfl_xor(v, m, 64));
  return v;
}

struct MinMaxArgs {
  PtrArr grads;
  PtrArr efs;
  float* pmin;       // n * (d >> L1)
  float* pmax;
  uint64_t d;
  uint32_t L1;       // log2 of min(B, 8192)
};

template <bool BF16, bool EF>
__global__ __launch_bounds__(NT) void k_minmax(const MinMaxArgs a) {
  __shared__ float smin[32], smax[32];   // one per 256 consecutive coordinates of the tile
  const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
  const uint32_t worker = blockIdx.y;
  const uint64_t off = (uint64_t)xcd_tile(blockIdx.x, gridDim.x) << LOG_TILE;
  const float* ef = EF ? static_cast<const float*>(a.efs.p[worker]) : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint64_t j = off + 4u * (uint32_t)(i * NT + t);
    float mn = __builtin_inff(), mx = -__builtin_inff();
    if (j < a.d) {
      float4 x = load_grad4<BF16>(a.grads.p[worker], j);
      if constexpr (EF) {
        const float4 e = *reinterpret_cast<const float4*>(ef + j);
        x.x += e.x; x.y += e.y; x.z += e.z; x.w += e.w;
      }
      mn = __builtin_fminf(__builtin_fminf(x.x, x.y), __builtin_fminf(x.z, x.w));
      mx = __builtin_fmaxf(__builtin_fmaxf(x.x, x.y), __builtin_fmaxf(x.z, x.w));
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if (lane == 0) { smin[i * 8 + wave] = mn; smax[i * 8 + wave] = mx; }
  }
  __syncthreads();
  const int nblk = TILE >> a.L1, cpb = 32 / nblk;   // chunks of 256 per block inside the tile
  if (t < nblk) {
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int c = 0; c < cpb; ++c) {
      mn = __builtin_fminf(mn, smin[t * cpb + c]);
      mx = __builtin_fmaxf(mx, smax[t * cpb + c]);
    }
    const uint64_t pidx = (off >> a.L1) + t;
    if (pidx < (a.d >> a.L1)) {
      a.pmin[(uint64_t)worker * (a.d >> a.L1) + pidx] = mn;
      a.pmax[(uint64_t)worker * (a.d >> a.L1) + pidx] = mx;
    }
  }
}

struct MinMaxFinalArgs {
  const float* pmin;
  const float* pmax;
  float* range_m;
  float* range_M;
  uint64_t d;
  uint32_t n, L, L1;
};

__global__ __launch_bounds__(64) void k_minmax_final(const MinMaxFinalArgs a) {
  const uint64_t k = blockIdx.x;
  const int lane = threadIdx.x;
  const uint32_t ppb = 1u << (a.L - a.L1);
  const uint64_t per_worker = a.d >> a.L1;
  float mn = __builtin_inff(), mx = -__builtin_inff();
  for (uint32_t i = 0; i < a.n; ++i) {
    const uint64_t base = (uint64_t)i * per_worker + k * ppb;
    for (uint32_t j = lane; j < ppb; j += 64) {
      mn = __builtin_fminf(mn, a.pmin[base + j]);
      mx = __builtin_fmaxf(mx, a.pmax[base + j]);
    }
  }
  mn = wave_min(mn);
  mx = wave_max(mx);
  if (lane == 0) { a.range_m[k] = mn; a.range_M[k] = mx; }
}

// Last strided pass of a forward RHT that keeps the rotated vector: finishes the butterflies, scales by
// 1/sqrt(B), writes the result back in place and records the tile's minimum and maximum.
struct HiStoreArgs {
  float* x;          // one worker's half-rotated vector, d floats, rotated in place
  float* pmin;       // this worker's partial minima, d >> L1 floats
  float* pmax;
  uint64_t d;
  TileMap tm;
  uint32_t L;
  float c;
};

template <int R>
__global__ __launch_bounds__(NT) void k_fwd_hi_store(const HiStoreArgs a) {
  __shared__ __align__(16) float lds[TILE];
  __shared__ float smin[16], smax[16];
  const int t = threadIdx.x, wave = t >> 6, lane = t & 63;
  const HiGeom<R> g(blockIdx.x, a.tm);
  if constexpr (R >= 2) {
    hi_front<R>(a.x, g, lds, t);
    int idx[2];
    float v[2][8];
    hi_back<R>(lds, t, idx, v);
    float mn = __builtin_inff(), mx = -__builtin_inff();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        v[h][e] *= a.c;
        mn = __builtin_fminf(mn, v[h][e]);
        mx = __builtin_fmaxf(mx, v[h][e]);
      }
      float* o = a.x + g.coord(idx[h]);
      *reinterpret_cast<float4*>(o) = make_float4(v[h][0], v[h][1], v[h][2], v[h][3]);
      *reinterpret_cast<float4*>(o + 4) = make_float4(v[h][4], v[h][5], v[h][6], v[h][7]);
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    if (lane == 0) { smin[wave] = mn; smax[wave] = mx; }
    __syncthreads();
    if (t == 0) {   // the whole tile lies in one block: one partial per tile
      for (int w = 1; w < 8; ++w) { mn = __builtin_fminf(mn, smin[w]); mx = __builtin_fmaxf(mx, smax[w]); }
      a.pmin[blockIdx.x] = mn;
      a.pmax[blockIdx.x] = mx;
    }
  } else {
    hi_load_to_lds<R>(a.x, g, a.d, lds, t);
    lds_stages<LOG_TILE - R, LOG_TILE, false, PLAIN>(lds, t, [](int, int, float) {});
    __syncthreads();
    // thread owns tile indices [8(t + 512h), +8): a wave covers 512 consecutive values per h
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int idx = 8 * (t + NT * h);
      const uint64_t j = g.coord(idx);
      float mn = __builtin_inff(), mx = -__builtin_inff();
      if (j < a.d) {
        float4 p0 = *reinterpret_cast<const float4*>(&lds[idx]);
        float4 p1 = *reinterpret_cast<const float4*>(&lds[idx + 4]);
        p0.x *= a.c; p0.y *= a.c; p0.z *= a.c; p0.w *= a.c;
        p1.x *= a.c; p1.y *= a.c; p1.z *= a.c; p1.w *= a.c;
        *reinterpret_cast<float4*>(a.x + j) = p0;
        *reinterpret_cast<float4*>(a.x + j + 4) = p1;
        mn = __builtin_fminf(__builtin_fminf(__builtin_fminf(p0.x, p0.y), __builtin_fminf(p0.z, p0.w)),
                             __builtin_fminf(__builtin_fminf(p1.x, p1.y), __builtin_fminf(p1.z, p1.w)));
        mx = __builtin_fmaxf(__builtin_fmaxf(__builtin_fmaxf(p0.x, p0.y), __builtin_fmaxf(p0.z, p0.w)),
                             __builtin_fmaxf(__builtin_fmaxf(p1.x, p1.y), __builtin_fmaxf(p1.z, p1.w)));
      }
      mn = wave_min(mn);
      mx = wave_max(mx);
      if (lane == 0) { smin[h * 8 + wave] = mn; smax[h * 8 + wave] = mx; }
    }
    __syncthreads();
    // blocks inside the tile (B < 8192) or the single one (then R rows of one block share the tile)
    const uint32_t L1 = a.L < LOG_TILE ? a.L : LOG_TILE;
    const int nblk = TILE >> L1, cpb = 16 / nblk;    // chunks of 512 per block inside the tile
    if (t < nblk) {
      float mn = __builtin_inff(), mx = -__builtin_inff();
      for (int c = 0; c < cpb; ++c) {
        mn = __builtin_fminf(mn, smin[t * cpb + c]);
        mx = __builtin_fmaxf(mx, smax[t * cpb + c]);
      }
      const uint64_t pidx = ((uint64_t)blockIdx.x << (LOG_TILE - L1)) + t;
      if (pidx < (a.d >> L1)) { a.pmin[pidx] = mn; a.pmax[pidx] = mx; }
    }
  }
}

// Uniform stochastic quantization of one worker's vector: 8192 consecutive coordinates per workgroup.
// Source: the rotated vector `x` when given, else grad (+ e).  Without rotation the error-feedback update
// e <- x - (m + z (M-m)/g) is done here; with rotation it needs an inverse transform (separate passes).
struct UQuantArgs {
  const float* x;          // rotated vector or null
  const void* grad;
  float* ef;               // error feedback, read (and written when ef_update) or null
  const float* range_M;
  const float* range_m;
  uint8_t* packed;
  uint64_t d;
  uint32_t L, b, g;
  uint32_t round, worker, k0, k1;
  uint32_t ef_update;
  uint64_t j0;             // global coordinate of the first element
  uint32_t lut[256];
};

template <bool BF16>
__global__ __launch_bounds__(NT) void k_uniform_quant(const UQuantArgs a) {
  __shared__ uint4 lut[256];
  __shared__ QuantScalars sQ[8];
  __shared__ int sWide[8];
  __shared__ float sStep[8];
  const int t = threadIdx.x;
  const uint64_t off = (uint64_t)xcd_tile(blockIdx.x, gridDim.x) << LOG_TILE;
  if (t < 256) {
    lut[t] = quant_lut_entry(a.lut[t]);
  }
  const int nblk = a.L < LOG_TILE ? (TILE >> a.L) : 1;
  if (t < nblk) {
    const uint64_t blk = (off >> a.L) + t;
    float M = 0.f, m = 0.f;
    if (blk < (a.d >> a.L)) { M = a.range_M[blk]; m = lower_of(a.range_m, blk, M); }
    bool wide;
    sQ[t] = quant_scalars(M, m, a.g, 1.0f, false, wide);
    sWide[t] = wide;
    sStep[t] = (float)(((double)M - (double)m) / (double)a.g);
  }
  __syncthreads();
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int idx = 8 * (t + NT * h);
    const uint64_t j = off + idx;
    if (j >= a.d) continue;
    float4 p0, p1;
    if (a.x) {
      p0 = *reinterpret_cast<const float4*>(a.x + j);
      p1 = *reinterpret_cast<const float4*>(a.x + j + 4);
    } else {
      p0 = load_grad4<BF16>(a.grad, j);
      p1 = load_grad4<BF16>(a.grad, j + 4);
      if (a.ef) {
        const float4 e0 = *reinterpret_cast<const float4*>(a.ef + j);
        const float4 e1 = *reinterpret_cast<const float4*>(a.ef + j + 4);
        p0.x += e0.x; p0.y += e0.y; p0.z += e0.z; p0.w += e0.w;
        p1.x += e1.x; p1.y += e1.y; p1.z += e1.z; p1.w += e1.w;
      }
    }
    const float hv[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
    const int bt = a.L < LOG_TILE ? (idx >> a.L) : 0;
    const QuantScalars s = sQ[bt];
    const uint64_t q = (a.j0 + j) >> 3;
    const uint4 rnd = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), a.round, a.worker, a.k0, a.k1);
    uint32_t z[8];
    if (!sWide[bt]) quantize8<true>(hv, rnd, s, lut, z);   // no scaling: the values are final (c = 1)
    else quantize8<true, true>(hv, rnd, s, lut, z);
    store_packed8(a.packed, j, a.b, z);
    if (a.ef_update) {
      const float step = sStep[bt], lo = s.lo;
      float e[8];
#pragma unroll
      for (int k = 0; k < 8; ++k) e[k] = hv[k] - ((float)z[k] * step + lo);   // identity table: T[z] = z
      *reinterpret_cast<float4*>(a.ef + j) = make_float4(e[0], e[1], e[2], e[3]);
      *reinterpret_cast<float4*>(a.ef + j + 4) = make_float4(e[4], e[5], e[6], e[7]);
    }
  }
}

// Alg. 1's estimate without rotation: out = m + X (M-m)/(g n), sixteen coordinates per thread.
struct UDequantArgs {
  const void* agg;
  const float* range_M;
  const float* range_m;
  float* out;
  uint64_t d;
  uint32_t L, agg_bits, divisor;
};

__global__ __launch_bounds__(256) void k_uniform_dequant(const UDequantArgs a) {
  if (a.agg_bits == 8 || a.agg_bits == 16) {
    // byte-aligned sums: four coordinates per thread and step, so that a wave writes 1 KB at a time
    const uint64_t base = (uint64_t)blockIdx.x * 4096;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint64_t j = base + 1024u * k + 4u * threadIdx.x;
      if (j >= a.d) return;
      uint32_t y[4];
      if (a.agg_bits == 8) {
        const uint32_t c = *reinterpret_cast<const uint32_t*>(static_cast<const uint8_t*>(a.agg) + j);
        y[0] = c & 255u; y[1] = (c >> 8) & 255u; y[2] = (c >> 16) & 255u; y[3] = c >> 24;
      } else {
        const uint2 c = *reinterpret_cast<const uint2*>(static_cast<const uint8_t*>(a.agg) + 2 * j);
        y[0] = c.x & 0xFFFFu; y[1] = c.x >> 16; y[2] = c.y & 0xFFFFu; y[3] = c.y >> 16;
      }
      const uint64_t blk = j >> a.L;
      const float M = a.range_M[blk], m = lower_of(a.range_m, blk, M);
      const float step = (float)(((double)M - (double)m) / (double)a.divisor);
      *reinterpret_cast<float4*>(a.out + j) =
          make_float4((float)y[0] * step + m, (float)y[1] * step + m, (float)y[2] * step + m, (float)y[3] * step + m);
    }
    return;
  }
  const uint64_t j = ((uint64_t)blockIdx.x * 256 + threadIdx.x) * 16;
  if (j >= a.d) return;
  uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0}, y[16];
  codes_load(static_cast<const uint8_t*>(a.agg), a.agg_bits, j, w, y);
  codes_decode(a.agg_bits, true, w, y);
  const uint64_t blk = j >> a.L;
  const float M = a.range_M[blk], m = lower_of(a.range_m, blk, M);
  const float step = (float)(((double)M - (double)m) / (double)a.divisor);
  float v[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) v[e] = (float)y[e] * step + m;
#pragma unroll
  for (int e = 0; e < 16; e += 4)
    *reinterpret_cast<float4*>(a.out + j + e) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);
}

}  // namespace thc
