// Stand-alone measurements of the hardware facts the THC kernels' tiling relies on (MI355X, gfx950).
// Not part of libthc: build with
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops access_patterns.hip -o access_patterns
// and run without arguments (needs about 9 GB of device memory, a few seconds).
//
//   1. tiles      copy / pack kernels that touch memory like the transform passes do: a workgroup owns a tile of
//                 2^R rows of 2^W consecutive floats; which offset bits are the row index and which bits the low
//                 three bits of the workgroup id (= its XCD, ids are dealt round-robin to the 8 XCDs) select.
//   2. chain      a copy followed by an 8:1 reduction of what it wrote, over the whole vector or piece by piece
//                 through one reused intermediate: what the 256 MB memory-side cache is worth between two kernels,
//                 and what a dependent launch costs.
//   3. valu       wave64 instructions per second per SIMD for independent chains of four instruction kinds.
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                      \
  do {                                                                             \
    hipError_t e_ = (x);                                                           \
    if (e_ != hipSuccess) {                                                        \
      std::printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__);   \
      std::exit(1);                                                                \
    }                                                                              \
  } while (0)

static hipEvent_t e0, e1;

template <class F>
static float time_ms(F launch, int reps = 5) {
  launch();
  launch();
  CK(hipEventRecord(e0));
  for (int i = 0; i < reps; ++i) launch();
  CK(hipEventRecord(e1));
  CK(hipEventSynchronize(e1));
  CK(hipGetLastError());
  float ms;
  CK(hipEventElapsedTime(&ms, e0, e1));
  return ms / reps;
}

// ---------------------------------------------------------------------------------------------- 1. tiles
struct Map {
  uint32_t rowpos, xpos, R, W;   // row index at offset bits [rowpos, rowpos + R), XCD bits at [xpos, xpos + 3)
  uint32_t freepos[32], nfree;   // where the remaining bits of the workgroup id go, low to high
};

template <int NT, bool PACK>
__global__ __launch_bounds__(NT) void k_tile(const float* __restrict__ x, float* __restrict__ y, Map m) {
  const uint32_t tile = blockIdx.x;
  uint64_t base = (uint64_t)(tile & 7u) << m.xpos;
  uint32_t rest = tile >> 3;
  for (uint32_t i = 0; i < m.nfree; ++i) {
    base |= (uint64_t)(rest & 1u) << m.freepos[i];
    rest >>= 1;
  }
  const int t = threadIdx.x;
  float4 v[4];
  uint64_t a[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t idx = 4u * (i * NT + t);
    a[i] = base + ((uint64_t)(idx >> m.W) << m.rowpos) + (idx & ((1u << m.W) - 1u));
    v[i] = *reinterpret_cast<const float4*>(x + a[i]);
  }
  if (PACK) {   // 4 bits per coordinate out, like the quantizer: eight coordinates -> four bytes
#pragma unroll
    for (int i = 0; i < 4; i += 2) {
      const float s = v[i].x + v[i].y + v[i].z + v[i].w + v[i + 1].x;
      const uint32_t idx = 8u * ((i / 2) * NT + t);
      const uint64_t c = base + ((uint64_t)(idx >> m.W) << m.rowpos) + (idx & ((1u << m.W) - 1u));
      *reinterpret_cast<uint32_t*>(reinterpret_cast<uint8_t*>(y) + (c >> 1)) = __float_as_uint(s);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<float4*>(y + a[i]) = v[i];
  }
}

static void run_tile(const float* x, float* y, int logd, int lt, uint32_t R, uint32_t rowpos, uint32_t xpos, bool pack) {
  Map m{};
  m.R = R;
  m.W = lt - R;
  m.rowpos = rowpos;
  m.xpos = xpos;
  bool used[40] = {};
  for (uint32_t b = 0; b < m.W; ++b) used[b] = true;
  for (uint32_t b = 0; b < R; ++b) used[rowpos + b] = true;
  for (uint32_t b = 0; b < 3; ++b) {
    if (used[xpos + b]) { std::printf("  (skipped: XCD bits overlap the tile)\n"); return; }
    used[xpos + b] = true;
  }
  for (uint32_t b = 0; b < (uint32_t)logd; ++b)
    if (!used[b]) m.freepos[m.nfree++] = b;
  const unsigned tiles = 1u << (logd - lt);
  const float ms = time_ms([&] {
    if (lt == 13) {
      if (pack) k_tile<512, true><<<tiles, 512>>>(x, y, m); else k_tile<512, false><<<tiles, 512>>>(x, y, m);
    } else {
      if (pack) k_tile<1024, true><<<tiles, 1024>>>(x, y, m); else k_tile<1024, false><<<tiles, 1024>>>(x, y, m);
    }
  });
  const double bytes = (double)(1ull << logd) * (pack ? 4.5 : 8.0);
  std::printf("  tile 2^%d = %4u rows x %5u B, rows at bit %2u, XCD at bit %2u, %s: %7.3f ms %6.2f TB/s\n", lt, 1u << R,
              4u << m.W, rowpos, xpos, pack ? "pack" : "copy", ms, bytes / ms / 1e9);
  std::fflush(stdout);
}

// ---------------------------------------------------------------------------------------------- 2. chain
__global__ __launch_bounds__(256) void k_copy(const float4* __restrict__ x, float4* __restrict__ y, uint64_t n) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) y[i] = x[i];
}

__global__ __launch_bounds__(256) void k_reduce8(const float4* __restrict__ x, float4* __restrict__ y, uint64_t nout) {
  const uint64_t o = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  if (o >= nout) return;
  const uint64_t blk = (uint64_t)blockIdx.x * 2048;
  float4 s = make_float4(0, 0, 0, 0);
#pragma unroll
  for (int k = 0; k < 8; ++k) {
    const float4 v = x[blk + k * 256 + threadIdx.x];
    s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
  }
  y[o] = s;
}

// ---------------------------------------------------------------------------------------------- 3. valu
template <int MODE>
__global__ __launch_bounds__(512) void k_valu(float* out, int iters, float a, float b) {
  float x[8];
  uint32_t u[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) { x[i] = threadIdx.x * 0.001f + i; u[i] = threadIdx.x * 2654435761u + i; }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 8; ++r) {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if (MODE == 0) x[i] = __builtin_fmaf(x[i], a, b);
        else if (MODE == 1) x[i] = x[i] + a;
        else if (MODE == 2) { const uint64_t p = (uint64_t)u[i] * 0xD2511F53u; u[i] = (uint32_t)p ^ (uint32_t)(p >> 32); }
        else u[i] = __builtin_amdgcn_bitop3_b32(u[i], u[(i + 1) & 7], 0x9E3779B9u, 0x96);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i) s += x[i] + (float)u[i];
  if (s == 1.2345f) out[0] = s;
}

template <int MODE>
static void run_valu(const char* name, float* out, double per_iter) {
  const unsigned grid = 256 * 4 * 4;   // 4 workgroups of 8 waves per CU, 4 rounds
  const int iters = 2000;
  const float ms = time_ms([&] { k_valu<MODE><<<grid, 512>>>(out, iters, 1.0001f, 0.5f); }, 1);
  const double insts = grid * 8.0 * iters * per_iter;
  std::printf("  %-22s %8.3f ms  %.3f G wave-instructions/s per SIMD (1024 SIMDs)\n", name, ms, insts / (ms * 1e-3) / 1024 / 1e9);
}

int main() {
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  const int logd = 30;                 // floats per buffer: 4 GiB
  const uint64_t d = 1ull << logd;
  float *x, *y;
  CK(hipMalloc(&x, d * 4));
  CK(hipMalloc(&y, d * 4));
  CK(hipMemset(x, 0, d * 4));

  std::printf("1. tiles (copy = 4 B in + 4 B out per float, pack = 4 B in + 0.5 B out)\n");
  std::printf(" first pass, 8192 consecutive floats per workgroup, XCD bits at 13 .. 20:\n");
  for (uint32_t xp = 13; xp <= 20; ++xp) run_tile(x, y, logd, 13, 0, 13, xp, false);
  std::printf(" first pass, 8 rows of 4 KB (rows at bits 13..15 or 16..18), XCD bits below the rows:\n");
  run_tile(x, y, logd, 13, 3, 13, 10, false);
  run_tile(x, y, logd, 13, 3, 16, 10, false);
  run_tile(x, y, logd, 14, 4, 13, 10, false);
  std::printf(" strided passes, R row bits at the top of a 2^20 block:\n");
  for (int pack = 0; pack < 2; ++pack) {
    run_tile(x, y, logd, 13, 4, 16, 10, pack);
    run_tile(x, y, logd, 13, 5, 15, 10, pack);
    run_tile(x, y, logd, 13, 6, 14, 10, pack);
    run_tile(x, y, logd, 13, 7, 13, 10, pack);
    run_tile(x, y, logd, 13, 7, 13, 6, pack);
    run_tile(x, y, logd, 13, 8, 12, 9, pack);
    run_tile(x, y, logd, 13, 9, 11, 8, pack);
    run_tile(x, y, logd, 14, 7, 13, 10, pack);
  }

  std::printf("2. chain: copy, then 8:1 reduce of the copy (4 GiB in, intermediate 4 GiB or one reused piece)\n");
  {
    const uint64_t total = d / 4;      // float4
    float4* X = reinterpret_cast<float4*>(x);
    float4* T = reinterpret_cast<float4*>(y);
    float4* O;
    CK(hipMalloc(&O, total * 2));
    auto chain = [&](uint64_t piece, bool reuse) {
      const uint64_t np = total / piece;
      const float ms = time_ms([&] {
        for (uint64_t c = 0; c < np; ++c) {
          float4* t = reuse ? T : T + c * piece;
          k_copy<<<(unsigned)(piece / 256), 256>>>(X + c * piece, t, piece);
          k_reduce8<<<(unsigned)(piece / 8 / 256), 256>>>(t, O + c * (piece / 8), piece / 8);
        }
      });
      std::printf("  piece %5.0f MB, %s, %4llu launches: %7.3f ms  %5.2f TB/s over the fabric\n", piece * 16.0 / 1048576,
                  reuse ? "one reused intermediate " : "intermediate of its own ", (unsigned long long)(2 * np), ms,
                  (total * 16.0 * 3 + total * 2.0) / ms / 1e9);
      std::fflush(stdout);
    };
    chain(total, false);
    for (uint64_t mb : {512ull, 256ull, 128ull, 64ull, 32ull, 16ull}) {
      chain(mb * 65536, false);
      chain(mb * 65536, true);
    }
    CK(hipFree(O));
  }

  std::printf("3. valu (independent chains, 8 waves per SIMD)\n");
  run_valu<0>("v_fma_f32", x, 64);
  run_valu<1>("v_add_f32", x, 64);
  run_valu<2>("v_mad_u64_u32 + v_xor", x, 128);
  run_valu<3>("v_bitop3_b32", x, 64);
  return 0;
}
