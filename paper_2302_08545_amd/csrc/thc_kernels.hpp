// THC hot-path kernels for gfx950.  See include/thc.h for the conventions (streams, bit order, RNG).
//
// A Hadamard transform of a block of B = 2^L coordinates is split by index bits:
//   "lo"  pass: bits [0, L1), L1 = min(L, 13): one workgroup owns 8192 consecutive coordinates
//   "mid" pass: (only for L > 22) up to 7 more bits each, in place in the workspace
//   "hi"  pass: the remaining bits (at most 9): one workgroup owns 2^R rows, 8192 >> R consecutive
//               coordinates wide
// Which bits each pass takes, and in which order, is fixed by the stage order (thc_params.stage_order) and
// reaches the kernels as TileMap tables; the rounding of every butterfly is therefore fixed.
//
//   thc_device.hpp     building blocks: tiling, Philox, butterflies, LDS rounds, bit-stream codec
//   thc_forward.hpp    k_fwd_lo, k_range, k_mid, k_fwd_hi_quant
//   thc_inverse.hpp    k_inv_lo, k_inv_hi
//   thc_uniform.hpp    k_minmax, k_minmax_final, k_fwd_hi_store, k_uniform_quant, k_uniform_dequant
//   thc_aggregate.hpp  k_aggregate_b4w8, k_aggregate_b4w16, k_aggregate_b2w8, k_aggregate_generic
//   thc_pipeline.hpp   k_pipe_forward: the forward passes of all blocks in one launch, block after block
#pragma once

#include "thc_forward.hpp"
#include "thc_inverse.hpp"
#include "thc_uniform.hpp"
#include "thc_aggregate.hpp"
#include "thc_pipeline.hpp"
