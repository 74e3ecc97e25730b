// Inverse transform passes: decompression and the error-feedback update (Alg. 2 / Alg. 3).
#pragma once

#include "thc_forward.hpp"

namespace thc {

// ---------------------------------------------------------------------------------------------
// Sixteen consecutive codes (table indices or aggregated sums) of `bits` bits each, starting at
// coordinate j (a multiple of 16): codes_load fetches the raw words (for the widths with a fast path)
// or the decoded fields (any other width); codes_decode finishes the fast paths.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void codes_load(const uint8_t* s8, uint32_t bits, uint64_t j, uint32_t (&w)[8],
                                           uint32_t (&y)[16]) {
  if (bits == 8) {
    const uint4 r = *reinterpret_cast<const uint4*>(s8 + j);
    w[0] = r.x; w[1] = r.y; w[2] = r.z; w[3] = r.w;
  } else if (bits == 16) {
    const uint4 r0 = *reinterpret_cast<const uint4*>(s8 + 2 * j);
    const uint4 r1 = *reinterpret_cast<const uint4*>(s8 + 2 * j + 16);
    w[0] = r0.x; w[1] = r0.y; w[2] = r0.z; w[3] = r0.w; w[4] = r1.x; w[5] = r1.y; w[6] = r1.z; w[7] = r1.w;
  } else if (bits == 4) {
    const uint2 r = *reinterpret_cast<const uint2*>(s8 + (j >> 1));
    w[0] = r.x; w[1] = r.y;
  } else if (bits == 2) {
    w[0] = *reinterpret_cast<const uint32_t*>(s8 + (j >> 2));
  } else if (bits == 1) {
    w[0] = *reinterpret_cast<const uint16_t*>(s8 + (j >> 3));
  } else {   // any other width: eight fields take `bits` bytes
    uint32_t z0[8], z1[8];
    load_fields8(s8 + (j >> 3) * bits, bits, z0);
    load_fields8(s8 + ((j >> 3) + 1) * bits, bits, z1);
#pragma unroll
    for (int e = 0; e < 8; ++e) { y[e] = z0[e]; y[8 + e] = z1[e]; }
  }
}

// Sixteen W-bit fields out of a staged bit stream: they start at `first`, or 16 bits into it (`half`).  W is a
// compile-time constant so that every field's word and shift are; one dword of slack is read past the fields.
template <int W>
__device__ __forceinline__ void cut16(const uint32_t* first, bool half, uint32_t (&y)[16]) {
  constexpr int NW = (16 * W + 31) / 32;          // dwords the fields span when they start on a boundary
  uint32_t d[NW + 1];
#pragma unroll
  for (int k = 0; k <= NW; ++k) d[k] = first[k];
  if (half) {
#pragma unroll
    for (int k = 0; k < NW; ++k) d[k] = __builtin_amdgcn_alignbit(d[k + 1], d[k], 16);
  }
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    constexpr uint32_t mask = (1u << W) - 1u;
    const int k = (e * W) >> 5, sh = (e * W) & 31;
    uint32_t v = d[k] >> sh;
    if (sh + W > 32) v |= d[k + 1] << (32 - sh);
    y[e] = v & mask;
  }
}

// widths that codes_load / codes_decode take straight from global memory
__device__ __forceinline__ bool codes_fast_width(uint32_t bits) {
  return bits == 8 || bits == 16 || bits == 4 || bits == 2 || bits == 1;
}

__device__ __forceinline__ void codes_decode(uint32_t bits, bool ok, const uint32_t (&w)[8], uint32_t (&y)[16]) {
  if (bits == 8) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (w[e >> 2] >> (8 * (e & 3))) & 255u;
  } else if (bits == 16) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (w[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
  } else if (bits == 4) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (w[e >> 3] >> (4 * (e & 7))) & 15u;
  } else if (bits == 2) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (w[0] >> (2 * e)) & 3u;
  } else if (bits == 1) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = (w[0] >> e) & 1u;
  } else if (!ok) {
#pragma unroll
    for (int e = 0; e < 16; ++e) y[e] = 0;
  }
}

// ---------------------------------------------------------------------------------------------
// Inverse "lo" pass.  Source is either the aggregated stream (decompression, Alg. 2:
// m + (Y/n)(M-m)/g = Y * step_n - M) or one worker's packed indices (error feedback, Alg. 3:
// X_i = m + T[z](M-m)/g = T[z] * step_g - M).  One thread loads 16 consecutive coordinates.
// ---------------------------------------------------------------------------------------------
struct InvLoArgs {
  PtrArr src;              // per vector of the launch (grid.y): aggregated stream or packed indices
  const float* range_M;
  const float* range_m;    // or null: m = -M
  float* ws_x;             // d floats per vector of the launch, written
  uint64_t d;
  uint32_t L;
  uint32_t src_bits;       // bits per coordinate in src
  uint32_t use_table;      // 1: src holds table indices; 0: src holds aggregated table values
  uint32_t divisor;        // g*n (aggregated) or g (indices)
  TileMap tm;
  uint8_t table[256];
};

struct alignas(16) SmemInvLo {
  float lds[TILE];
  float sM[8], sStep[8];
  float tabf[256];
};

// One tile: tile index `tile` of the launch's vector `vec`; the results go to dst_vec[offset in the vector].
template <int L1, bool XO, class A>
__device__ __forceinline__ void inv_lo_tile(const A& a, uint32_t tile, uint32_t vec, float* dst_vec,
                                            SmemInvLo& sm) {
  static_assert(!XO || L1 == LOG_TILE, "the row-split tile needs blocks of at least 2^16");
  constexpr bool GUARD = L1 < LOG_TILE;
  float* const lds = sm.lds;
  float* const sM = sm.sM;
  float* const sStep = sm.sStep;
  float* const tabf = sm.tabf;

  const int t = threadIdx.x;
  const uint64_t off = tm_base(a.tm, tile);
  const int idx = 16 * t;
  const uint64_t j = off + lo_map<XO>(idx);
  const bool ok = !GUARD || j < a.d;
  const uint8_t* const src = static_cast<const uint8_t*>(a.src.p[vec]);

  // raw bits first, so the load is in flight while the block constants are prepared
  uint32_t w[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  uint32_t y[16];
  const bool staged = !codes_fast_width(a.src_bits);
  if (!staged) {
    if (ok) codes_load(src, a.src_bits, j, w, y);
  } else {
    // Any other width: the tile's eight runs of 1024 codes (128 * bits bytes each, dword aligned) are copied
    // into the still unused tile buffer with coalesced loads; every thread then cuts its sixteen fields out.
    uint32_t* stage = reinterpret_cast<uint32_t*>(lds);
    const uint32_t per_row = 32u * a.src_bits;                       // dwords per 1024 codes: fewer than NT
    if ((uint32_t)t < per_row) {
      uint32_t val[8];
#pragma unroll
      for (uint32_t r = 0; r < 8; ++r) {
        const uint64_t jr = off + lo_map<XO>(1024u * r);             // first coordinate of the run
        val[r] = 0;
        if (!GUARD || jr < a.d)                                      // runs exist whole or not at all: 1024 divides d
          val[r] = reinterpret_cast<const uint32_t*>(src + (jr >> 3) * a.src_bits)[t];
      }
#pragma unroll
      for (uint32_t r = 0; r < 8; ++r) stage[r * per_row + t] = val[r];
    }
  }

  const int nblk = a.L < LOG_TILE ? (TILE >> a.L) : 1;
  if (t < nblk) {
    const uint64_t blk = (off >> a.L) + t;
    float M = 0.f, m = 0.f;
    if (blk < (a.d >> a.L)) { M = a.range_M[blk]; m = lower_of(a.range_m, blk, M); }
    sM[t] = m;                                                   // the affine map only needs the lower end
    sStep[t] = (float)(((double)M - (double)m) / (double)a.divisor);
  }
  if (a.use_table && t < 256) tabf[t] = (float)a.table[t];
  __syncthreads();

  if (!staged) {
    codes_decode(a.src_bits, ok, w, y);
  } else {
    // sixteen fields start at bit 16 * (field number / 16) * bits of the run: on a dword boundary or in its middle
    const uint32_t* stage = reinterpret_cast<const uint32_t*>(lds);
    const uint32_t pos = (uint32_t)(idx & 1023) * a.src_bits;
    const uint32_t* first = stage + (uint32_t)(idx >> 10) * 32u * a.src_bits + (pos >> 5);
    switch (a.src_bits) {
#define THC_CUT(W) case W: cut16<W>(first, (pos & 16u) != 0, y); break;
      THC_CUT(3) THC_CUT(5) THC_CUT(6) THC_CUT(7) THC_CUT(9) THC_CUT(10) THC_CUT(11) THC_CUT(12) THC_CUT(13)
      THC_CUT(14) THC_CUT(15)
#undef THC_CUT
      default: break;
    }
    if (!ok) {
#pragma unroll
      for (int e = 0; e < 16; ++e) y[e] = 0;
    }
    __syncthreads();                                                 // every field is out before the tile is written
  }
  const int bt = a.L < LOG_TILE ? (idx >> a.L) : 0;
  const float lo = sM[bt], step = sStep[bt];
  float v[16];
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const float f = a.use_table ? tabf[y[e]] : (float)y[e];
    v[e] = ok ? f * step + lo : 0.f;
  }
  bfly<4>(v);
#pragma unroll
  for (int e = 0; e < 16; e += 4)
    *reinterpret_cast<float4*>(&lds[swz(idx + e)]) = make_float4(v[e], v[e + 1], v[e + 2], v[e + 3]);

  float* dst = dst_vec + off;
  const uint64_t left = a.d - off;
  lds_stages<4, L1, true, SWZ>(lds, t, [&](int base, int eoff, float val) {
    if (!GUARD || (uint64_t)(base + eoff) < left) dst[lo_map<XO>(base) + lo_map<XO>(eoff)] = val;
  });
}

template <int L1, bool XO>
__global__ __launch_bounds__(NT) void k_inv_lo(const InvLoArgs a) {
  __shared__ SmemInvLo sm;
  inv_lo_tile<L1, XO>(a, blockIdx.x, blockIdx.y, a.ws_x + (uint64_t)blockIdx.y * a.d, sm);
}

// ---------------------------------------------------------------------------------------------
// Inverse "hi" pass: finish H, scale by 1/sqrt(B), apply the diagonal (Sec. 5.1: RHT^-1 = D H / sqrt(d)).
// mode 0: out = result (Alg. 3, the global update);
// mode 1: e <- (grad + e) - result (Alg. 3, error-feedback update), out = ef buffer, read and written.
// ---------------------------------------------------------------------------------------------
struct InvHiArgs {
  const float* x;      // half-rotated vectors, d floats per vector of the launch (grid.y)
  PtrArr out;          // per vector: d floats
  PtrArr grad;         // per vector, mode 1 only
  uint64_t d;
  uint64_t j0;         // global coordinate of x[0] (a multiple of B), for the diagonal's random stream
  TileMap tm;
  uint32_t round, k0, k1;
  uint32_t mode, bf16;
  float c;
};

// scale by 1/sqrt(B) and apply the diagonal; mode 1: (x + e) - that
template <class A>
__device__ __forceinline__ float4 inv_finish4(float4 v, uint32_t bits, const A& a, float4 x, float4 e) {
  v.x = flip(v.x * a.c, bits & 1u);
  v.y = flip(v.y * a.c, (bits >> 1) & 1u);
  v.z = flip(v.z * a.c, (bits >> 2) & 1u);
  v.w = flip(v.w * a.c, (bits >> 3) & 1u);
  if (a.mode == 1) {
    x.x += e.x; x.y += e.y; x.z += e.z; x.w += e.w;
    v = make_float4(x.x - v.x, x.y - v.y, x.z - v.z, x.w - v.w);
  }
  return v;
}

template <class A>
__device__ __forceinline__ float4 inv_finish4(float4 v, uint32_t bits, const A& a, const float* out,
                                              const void* grad, uint64_t j) {
  float4 x = make_float4(0.f, 0.f, 0.f, 0.f), e = x;
  if (a.mode == 1) {
    x = a.bf16 ? load_grad4<true>(grad, j) : load_grad4<false>(grad, j);
    e = *reinterpret_cast<const float4*>(out + j);
  }
  return inv_finish4(v, bits, a, x, e);
}

struct alignas(16) SmemInvHi {
  float lds[TILE];
  uint32_t sgn[TILE / 32];
};

// One tile: tile index `tile` of the launch's vector `vec`, whose half-rotated image starts at xv.
template <int R, class A>
__device__ __forceinline__ void inv_hi_tile(const A& a, uint32_t tile, uint32_t vec, const float* xv,
                                            SmemInvHi& sm) {
  float* const lds = sm.lds;
  uint32_t* const sgn = sm.sgn;

  const int t = threadIdx.x;
  const HiGeom<R> g(tile, a.tm);
  float* const out = static_cast<float*>(const_cast<void*>(a.out.p[vec]));
  const void* const grad = a.grad.p[vec];

  if constexpr (R >= 2) {
    float4 x[4];
    hi_issue_loads<R>(xv, g, t, x);
    // the diagonal's bits while the loads travel
    // 32 consecutive tile indices are 32 consecutive coordinates, or, with 16-wide rows, two aligned halves
    if (t < TILE / 32) {
      if constexpr (HiGeom<R>::W >= 32) {
        sgn[t] = sign_word(a.j0 + g.coord(32 * t), a.round, a.k0, a.k1);
      } else {
        const uint64_t j0 = a.j0 + g.coord(32 * t), j1 = a.j0 + g.coord(32 * t + 16);
        const uint32_t lo = sign_word(j0 & ~31ull, a.round, a.k0, a.k1) >> (j0 & 31);
        const uint32_t hi = sign_word(j1 & ~31ull, a.round, a.k0, a.k1) >> (j1 & 31);
        sgn[t] = (lo & 0xFFFFu) | (hi << 16);
      }
    }
    hi_r0_to_lds<R>(x, lds, t);
    hi_round1<R>(lds, t);
    int idx[2];
    hi_back_index<R>(t, idx);
    // error-feedback update: the gradient and the buffer's old contents are requested for both halves before
    // anything is stored (the stores go to that same buffer), and while the tile's last stage runs
    float4 gx[2][2], ex[2][2];
    if (a.mode == 1) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint64_t j = g.coord(idx[h]);
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          gx[h][k] = a.bf16 ? load_grad4<true>(grad, j + 4 * k) : load_grad4<false>(grad, j + 4 * k);
          ex[h][k] = *reinterpret_cast<const float4*>(out + j + 4 * k);
        }
      }
    } else {
#pragma unroll
      for (int h = 0; h < 2; ++h)
        for (int k = 0; k < 2; ++k) gx[h][k] = ex[h][k] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    float v[2][8];
    hi_back<R>(lds, t, idx, v);
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint64_t j = g.coord(idx[h]);
      const uint32_t bits = sgn[idx[h] >> 5] >> (idx[h] & 31);
      const float4 o0 = inv_finish4(make_float4(v[h][0], v[h][1], v[h][2], v[h][3]), bits, a, gx[h][0], ex[h][0]);
      const float4 o1 = inv_finish4(make_float4(v[h][4], v[h][5], v[h][6], v[h][7]), bits >> 4, a, gx[h][1], ex[h][1]);
      *reinterpret_cast<float4*>(out + j) = o0;
      *reinterpret_cast<float4*>(out + j + 4) = o1;
    }
  } else {
    if (t < TILE / 32) sgn[t] = sign_word(a.j0 + g.coord(32 * t), a.round, a.k0, a.k1);
    hi_load_to_lds<R>(xv, g, a.d, lds, t);
    lds_stages<LOG_TILE - R, LOG_TILE, false, PLAIN>(lds, t, [](int, int, float) {});
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = 4 * (i * NT + t);
      const uint64_t j = g.coord(idx);
      if (j >= a.d) continue;
      const float4 v = *reinterpret_cast<const float4*>(&lds[idx]);
      const uint32_t bits = sgn[idx >> 5] >> (idx & 31);
      *reinterpret_cast<float4*>(out + j) = inv_finish4(v, bits, a, out, grad, j);
    }
  }
}

template <int R>
__global__ __launch_bounds__(NT) void k_inv_hi(const InvHiArgs a) {
  __shared__ SmemInvHi sm;
  inv_hi_tile<R>(a, blockIdx.x, blockIdx.y, a.x + (uint64_t)blockIdx.y * a.d, sm);
}

}  // namespace thc
