// The worker side of a round as ONE launch: the passes of the transform follow each other block by block inside
// the kernel instead of kernel by kernel over the whole vector (Alg. 3: RHT, range, clamp + SQ + index + pack,
// optional error-feedback update).
//
// Why.  A 2^20-point block (4 MB) does not fit one compute unit, so its transform takes two trips through memory
// with an intermediate in between.  Launch by launch that intermediate is as long as a group of blocks of all vectors
// (gigabytes).  Here a block's intermediate is read back a few hundred microseconds after it was written, from a ring
// of a few block-sized slots, and the memory-bound first pass of one block shares the compute units with the
// ALU-bound quantizer of another.  Measured on MI355X the sweep takes the same time either way (within 2 %: both
// forms run at what the fabric between the XCDs and memory delivers); what this form saves is workspace, a ring of
// 4 (8 with error feedback) blocks per vector instead of a group's worth.
//
// Order.  Work items are numbered so that everything an item waits for has a smaller number:
//   step s = 0, 1, ...:  [range item of unit s-1]  then, interleaved in groups of eight workgroups,
//                        phase 0 of unit s, phase 1 of unit s - lag, phase 2 of unit s - 2 lag, ...
// (unit = one block of all W vectors; phases: 0 first pass, 1 last pass + quantizer, and with error feedback
// 2 inverse first pass, 3 inverse last pass + update).  Workgroups are dispatched in index order, so a waiting
// workgroup only ever waits for workgroups that already run; every wait is bounded all the same and gives up by
// raising a status word that the caller can read (nothing hangs; the results are then invalid).
//
// Visibility.  On this chip every XCD has its own L2, which holds a producer's stores until they are written back,
// and consecutive workgroups are dealt to the eight XCDs in turn (from a starting XCD that differs from launch to
// launch, so a workgroup asks the hardware which XCD it is on).  Every group of eight consecutive workgroups belongs
// to one unit and phase, hence each XCD runs an eighth of a unit's producers.  They count in per XCD once their stores
// are acknowledged; the one that completes its XCD's count writes that L2 back (a release fence at agent scope) and
// reports; consumers wait for all eight reports, invalidate (an acquire fence at agent scope) and read.  Eight
// write-backs per unit instead of one per workgroup: a release fence per workgroup was measured at 4x to 30x the run
// time of the whole chain.  Were workgroups ever dealt differently, a count would stay short and the waits would
// time out into the status word: never a silent wrong result.
#pragma once

#include "thc_inverse.hpp"

namespace thc {

constexpr uint32_t NXCD = 8;
constexpr uint32_t SYNC_STRIDE = 64;                       // counters sit 256 bytes apart: polls of one never queue behind updates of another
constexpr uint32_t SYNC_PHASE = NXCD + 1;                  // per phase: eight tallies and the report count
constexpr uint32_t SYNC_READY = 4 * SYNC_PHASE;            // range of the unit is in place
constexpr uint32_t SYNC_DONE = SYNC_READY + 1;             // workgroups of the last phase that are through
constexpr uint32_t SYNC_PER_UNIT = (SYNC_DONE + 1) * SYNC_STRIDE;
constexpr uint32_t PIPE_WAIT_SPINS = 250000;               // about a second of waiting before a workgroup gives up

enum : uint32_t { PIPE_OK = 0, PIPE_TIMEOUT = 1 };

struct PipeArgs {
  PtrArr grads, efs, packed;   // W vectors: gradients, error-feedback buffers (or unused), packed outputs
  float* ring;                 // slots * W * B floats
  double* partials;            // W * pstride
  uint64_t pstride;
  float* range_M;              // K floats: written by the range items (compute_range) or given
  const uint32_t* lut;         // device copy of the quantizer's 256 grid-cell entries
  uint32_t* sync;              // K * SYNC_PER_UNIT counters, zeroed before the launch
  uint32_t* status;            // one word, zeroed before the launch
  uint64_t d, j0;
  TileMap lo_tm, hi_tm;
  uint32_t L, W, K, slots, lag, nphase, compute_range;
  uint32_t b, g, round, worker0, k0, k1, bf16;
  float c, t_p;
  uint8_t table[256];
};

struct LoView {
  const PtrArr& grads;
  const PtrArr& efs;
  double* partials;
  uint64_t pstride, d, j0;
  uint32_t round, k0, k1;
  const TileMap& tm;
};
struct QuantView {
  const float* range_M;
  const float* range_m;
  const PtrArr& packed;
  uint64_t d, j0;
  const TileMap& tm;
  uint32_t L, b, g, round, worker, k0, k1;
  float c;
  const uint32_t* lut;
};
struct InvLoView {
  const PtrArr& src;
  const float* range_M;
  const float* range_m;
  uint64_t d;
  uint32_t L, src_bits, use_table, divisor;
  const TileMap& tm;
  const uint8_t* table;
};
struct InvHiView {
  const PtrArr& out;
  const PtrArr& grad;
  uint64_t d, j0;
  const TileMap& tm;
  uint32_t round, k0, k1, mode, bf16;
  float c;
};

__device__ __forceinline__ uint32_t xcc_id() {
  return __builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 15u;   // hardware register XCC_ID, bits [3:0]
}

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Thread 0 waits until *c >= target (bounded; a time-out anywhere ends every other wait too), the workgroup
// learns the outcome through `flag`.  ACQUIRE: ends with the caches invalidated for the data the counter announces
// (not needed where the counter only says that a buffer may be overwritten).
template <bool ACQUIRE>
__device__ __forceinline__ bool pipe_wait(const uint32_t* c, uint32_t target, uint32_t* status, int* flag) {
  if (threadIdx.x == 0) {
    int ok = 0;
    for (uint32_t it = 0; it < PIPE_WAIT_SPINS; ++it) {
      if (ld_agent(c) >= target) { ok = 1; break; }
      if (ld_agent(status) & PIPE_TIMEOUT) break;
      __builtin_amdgcn_s_sleep(64);
    }
    if (!ok) __hip_atomic_fetch_or(status, PIPE_TIMEOUT, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (ACQUIRE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    *flag = ok;
  }
  __syncthreads();
  const bool ok = *flag != 0;
  __syncthreads();            // `flag` may be rewritten by the next wait
  return ok;
}

// The workgroup's stores are done: count it in for its XCD; whoever completes the count writes the XCD's L2 back
// and reports.
__device__ __forceinline__ void pipe_publish(uint32_t* unit_sync, uint32_t phase, uint32_t per_xcd) {
  __builtin_amdgcn_s_waitcnt(0);      // vmcnt(0) expcnt(0) lgkmcnt(0): this wave's stores are acknowledged by the L2
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t x = xcc_id() & (NXCD - 1);     // the XCD whose L2 holds this workgroup's stores
    uint32_t* c = unit_sync + (phase * SYNC_PHASE) * SYNC_STRIDE;
    const uint32_t old = __hip_atomic_fetch_add(c + x * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == per_xcd - 1) {
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      __hip_atomic_fetch_add(c + NXCD * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

constexpr size_t pipe_smem_bytes() {
  size_t m = sizeof(SmemLo);
  if (sizeof(SmemQuant) > m) m = sizeof(SmemQuant);
  if (sizeof(SmemInvLo) > m) m = sizeof(SmemInvLo);
  if (sizeof(SmemInvHi) > m) m = sizeof(SmemInvHi);
  if (sizeof(SmemRange) > m) m = sizeof(SmemRange);
  return m;
}

// Blocks of 2^(13+R) coordinates, split stage order (first pass on eight rows of 1024 coordinates), no middle pass.
template <int R, bool BF16, bool EF>
__global__ __launch_bounds__(NT, 8) void k_pipe_forward(const PipeArgs P) {
  constexpr bool CFOLD = ((LOG_TILE + R) & 1) == 0;
  __shared__ __align__(16) unsigned char raw[pipe_smem_bytes()];
  __shared__ int flag;

  const uint32_t TB = 1u << R;                         // tiles per block
  const uint32_t Tu = P.W << R;                        // workgroups per unit and phase
  const uint32_t x = blockIdx.x & (NXCD - 1);
  const uint32_t r = blockIdx.x >> 3;
  const uint32_t per_step = (Tu >> 3) * P.nphase + 1;  // groups of eight workgroups per step
  const uint32_t step = r / per_step, q = r - step * per_step;

  if (q == 0) {
    // ---- range item of unit step-1: M_k from the norms of all W vectors, once the first pass has reported
    if (x != 0 || step == 0 || step > P.K) return;
    const uint32_t u = step - 1;
    uint32_t* us = P.sync + (uint64_t)u * SYNC_PER_UNIT;
    if (!pipe_wait<true>(us + NXCD * SYNC_STRIDE, NXCD, P.status, &flag)) return;
    if (P.compute_range) {
      const float M = block_range(P.partials, P.pstride, P.W, TB, u, P.t_p, P.L, *reinterpret_cast<SmemRange*>(raw));
      if (threadIdx.x == 0) {
        P.range_M[u] = M;
        __builtin_amdgcn_s_waitcnt(0);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      }
    }
    if (threadIdx.x == 0)
      __hip_atomic_store(us + SYNC_READY * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return;
  }

  const uint32_t phase = (q - 1) % P.nphase;
  const uint32_t tu = (((q - 1) / P.nphase) << 3) | x;  // tile within the unit: vector w, tile tb of the block
  if (step < phase * P.lag) return;
  const uint32_t u = step - phase * P.lag;
  if (u >= P.K) return;
  const uint32_t w = tu >> R, tb = tu & (TB - 1);
  const uint32_t gt = (u << R) | tb;                    // tile index in the whole vector
  uint32_t* us = P.sync + (uint64_t)u * SYNC_PER_UNIT;
  // where coordinate 0 of vector w would sit if the ring slot of unit u were part of a whole vector
  const int64_t slot_at = (int64_t)(((uint64_t)(u % P.slots) * P.W + w) << (LOG_TILE + R));
  float* const vec = P.ring + (slot_at - (int64_t)((uint64_t)u << (LOG_TILE + R)));

  if (phase == 0) {
    if (u >= P.slots) {   // the slot's previous tenant must be through its last phase
      const uint32_t* old = P.sync + (uint64_t)(u - P.slots) * SYNC_PER_UNIT + SYNC_DONE * SYNC_STRIDE;
      if (!pipe_wait<false>(old, Tu, P.status, &flag)) return;
    }
    const LoView a{P.grads, P.efs, P.partials, P.pstride, P.d, P.j0, P.round, P.k0, P.k1, P.lo_tm};
    fwd_lo_tile<LOG_TILE, BF16, EF, true, false>(a, gt, w, vec, *reinterpret_cast<SmemLo*>(raw));
    pipe_publish(us, 0, Tu >> 3);
  } else if (phase == 1) {
    if (!pipe_wait<true>(us + SYNC_READY * SYNC_STRIDE, 1u, P.status, &flag)) return;
    const QuantView a{P.range_M, nullptr, P.packed, P.d, P.j0, P.hi_tm, P.L, P.b, P.g, P.round, P.worker0, P.k0, P.k1,
                      P.c, P.lut};
    hi_quant_tile<R, CFOLD>(a, gt, w, vec, *reinterpret_cast<SmemQuant*>(raw));
    if constexpr (EF) {
      pipe_publish(us, 1, Tu >> 3);
    } else {
      if (threadIdx.x == 0)   // every wave's loads from the slot came back before the tile's last barrier
        __hip_atomic_fetch_add(us + SYNC_DONE * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  } else if constexpr (EF) {
    if (phase == 2) {
      // X_i from the indices, inverse first pass into the slot the quantizer has finished with
      if (!pipe_wait<true>(us + (1 * SYNC_PHASE + NXCD) * SYNC_STRIDE, NXCD, P.status, &flag)) return;
      const InvLoView a{P.packed, P.range_M, nullptr, P.d, P.L, P.b, 1u, P.g, P.lo_tm, P.table};
      inv_lo_tile<LOG_TILE, true>(a, gt, w, vec, *reinterpret_cast<SmemInvLo*>(raw));
      pipe_publish(us, 2, Tu >> 3);
    } else {
      // e <- (grad + e) - RHT^-1(X_i)
      if (!pipe_wait<true>(us + (2 * SYNC_PHASE + NXCD) * SYNC_STRIDE, NXCD, P.status, &flag)) return;
      const InvHiView a{P.efs, P.grads, P.d, P.j0, P.hi_tm, P.round, P.k0, P.k1, 1u, P.bf16, P.c};
      inv_hi_tile<R>(a, gt, w, vec, *reinterpret_cast<SmemInvHi*>(raw));
      if (threadIdx.x == 0)
        __hip_atomic_fetch_add(us + SYNC_DONE * SYNC_STRIDE, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// Before the launch: counters and status to zero, the quantizer's table entries into device memory.
struct PipeSetupArgs {
  uint32_t* sync;
  uint64_t nsync;
  uint32_t* status;
  uint32_t* lut_out;
  uint32_t lut[256];
};

__global__ __launch_bounds__(256) void k_pipe_setup(const PipeSetupArgs a) {
  const uint64_t i0 = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  for (uint64_t i = i0; i < a.nsync; i += (uint64_t)gridDim.x * 256) a.sync[i] = 0;
  if (blockIdx.x == 0) {
    a.lut_out[threadIdx.x] = a.lut[threadIdx.x];
    if (threadIdx.x == 0) *a.status = 0;
  }
}

}  // namespace thc
