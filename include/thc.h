/*
 * libthc -- Tensor Homomorphic Compression (arXiv 2302.08545), data-parallel hot path for AMD gfx950.
 *
 * One round of the paper's Alg. 3 ("Training with THC") maps onto four calls:
 *
 *   thc_prepare_range   preliminary stage: x_i = grad_i + e_i, per-block norms ||x_i||, the shared range
 *                       M_k = t_p * max_i ||x_i|| / sqrt(B), m_k = -M_k
 *   thc_compress        main stage, one worker: RHT, clamp to [-M, M], stochastic quantization onto the table's
 *                       grid, table index, bit-pack; optional error-feedback update
 *   thc_aggregate       main stage, parameter-server side: Y = sum_i T[Z_i] on the packed streams
 *   thc_decompress      worker side: m + (Y/n)(M-m)/g, then the inverse RHT
 *
 * and, for n workers whose buffers all live on one GPU, thc_compress_all does the work of thc_prepare_range and of
 * the n calls of thc_compress in one sweep that reads every gradient once (the paper runs the norm exchange and
 * the RHT side by side; here the norms come out of the transform's first pass).
 *
 * Conventions
 *   - All data pointers are DEVICE pointers (hipMalloc'd, 16-byte aligned) unless a comment says "host".
 *     Arrays of pointers (`grads`, `ef`, `packed`) are HOST arrays of device pointers.
 *   - `stream` is a hipStream_t passed as void*.  Every call validates its arguments on the host,
 *     enqueues its kernels on `stream` and returns without synchronizing.  Calls that share a workspace
 *     must be ordered on one stream (or by events).
 *   - The library allocates nothing and keeps no state, neither on the host nor in the workspace: workspace,
 *     range, error-feedback buffers, the round counter and the lookup table are owned by the caller, every call
 *     is complete by itself, and the workspace is scratch whose contents mean nothing between calls.  Inputs are
 *     never modified, except `ef_inout`.
 *   - Return value: THC_OK (0) or a negative thc_status.  Non-finite inputs (or inputs so large that their
 *     transform overflows binary32) are not detected; they propagate to unspecified (but in-bounds) results.
 *     A block whose scale g / (M - m), rounded to binary32, is not a finite number (M = m, or a width below
 *     about g * 2^-128) counts as empty: all its indices are 0 and it decodes to m (this covers the all-zero
 *     block, M = 0, which decodes to exact zeros).
 *   - Vector layout: a worker's gradient is one flat vector of d coordinates (padded by the caller with
 *     zeros to a multiple of `block`).  The RHT, the norm and the range are per block of `block`
 *     consecutive coordinates (the paper's 4 MB partition is block = 2^20).
 *   - Packed index stream and aggregated stream: bit streams of b-bit (agg_bits-bit) fields, field j at
 *     stream bits [j*w, j*w + w), stream bit k being bit (k mod 8) of byte (k div 8).  For agg_bits 8 / 16
 *     that is an array of little-endian uint8 / uint16.
 *   - Random numbers: Philox4x32-10 keyed by `seed`.  Rademacher diagonal D^r: coordinate j takes bit
 *     (j mod 32) of word ((j div 32) mod 4) of Philox(counter (q, q>>32, round, 0x80000000)), q = j div 128.
 *     Rounding draw of worker i: coordinate j takes 16-bit half (j mod 8) (low half first) of
 *     Philox(counter (q, q>>32, round, i)), q = j div 8; u = (half + 1/2) / 2^16.
 *     j is the coordinate's position in the whole vector: a call whose buffers hold only blocks
 *     [first_block, first_block + d/block) of a longer vector (a shard, a piece) sets thc_params.first_block
 *     and computes exactly what the call on the whole vector computes for those blocks.
 *   - Butterflies of the Hadamard transform run in the stage order of thc_params.stage_order, in binary32,
 *     without fused multiply-add; packed bytes and aggregated sums are therefore reproducible bit for bit.
 */
#ifndef THC_H_
#define THC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum thc_status {
  THC_OK = 0,
  THC_EINVAL = -1,       /* null or misaligned pointer, d/block/n/b/g out of range                         */
  THC_ETABLE = -2,       /* table is not 0 = T[0] < T[1] < ... < T[2^b-1] = g (homomorphism precondition)   */
  THC_EOVERFLOW = -3,    /* g*n does not fit in agg_bits                                                    */
  THC_EUNSUPPORTED = -4, /* valid in principle, not implemented (e.g. n > THC_MAX_WORKERS)                  */
  THC_ELAUNCH = -5       /* the HIP runtime rejected a launch; see hipGetLastError                          */
} thc_status;

enum { THC_MAX_WORKERS = 64 };
enum { THC_DTYPE_F32 = 0, THC_DTYPE_BF16 = 1 };

/* Order in which the butterfly stages of the Hadamard transform run (each stage pairs coordinates whose
 * offsets inside the block differ in one bit).  Every order computes the same transform; in binary32 the
 * roundings differ, so the order is part of what makes results reproducible bit for bit.
 *   THC_ORDER_ASCENDING  bits 0, 1, ..., log2(B)-1.
 *   THC_ORDER_SPLIT      for B >= 2^16: bits 0..9, 13, 14, 15, then 10, 11, 12, 16, ..., log2(B)-1 (the memory
 *                        access pattern of the first pass is faster on MI355X); same as ascending below 2^16. */
enum { THC_ORDER_ASCENDING = 0, THC_ORDER_SPLIT = 1 };

/* The problem statement of Alg. 3.  Plain data, owned by the caller, read on the host only. */
typedef struct thc_params {
  uint64_t d;          /* padded coordinate count per worker; a multiple of `block`, below 2^40            */
  uint64_t block;      /* B: RHT block, a power of two, 2^10 <= B <= 2^27, B divides d                     */
  uint32_t n;          /* number of workers, 1 <= n <= THC_MAX_WORKERS                                     */
  uint32_t b;          /* bits per table index, 1..8 (1, 2, 4, 8 have fast paths)                          */
  uint32_t g;          /* granularity: 2^b - 1 <= g <= 255 (Sec. 4.3)                                      */
  uint32_t agg_bits;   /* width of an aggregated value, 1..16 (8 and 16 have fast paths); g*n < 2^agg_bits */
  uint32_t in_dtype;   /* THC_DTYPE_F32 or THC_DTYPE_BF16 (widened to binary32 inside the kernel)          */
  float    t_p;        /* truncation threshold Phi^-1(1 - p/2) (Sec. 5.1); see thc_threshold               */
  uint64_t seed;       /* shared by all workers and the decompressor                                       */
  uint8_t  table[256]; /* T[0 .. 2^b-1]; see thc_solve_table                                               */
  uint32_t stage_order;/* THC_ORDER_ASCENDING or THC_ORDER_SPLIT                                           */
  uint32_t first_block;/* index, in the whole vector, of the first block these buffers hold (0 for a whole vector) */
  uint32_t group_log2; /* 0 = default (29).  The transform's passes walk a vector in groups of whole blocks of about
                          2^group_log2 coordinates (over all vectors of the call), 10..40: it sizes the workspace
                          (which therefore does not grow with d); never a result */
  uint32_t single_launch; /* 0 or 1.  1: thc_compress and thc_compress_all run all passes of all blocks in ONE kernel
                          launch where they can (split stage order, blocks of 2^17 .. 2^22, at least four blocks,
                          group_log2 = 0), blocks following each other through a ring of a few block-sized slots: a
                          sixteenth of the workspace at the same speed (within 2 %) without error feedback; with error
                          feedback and n * block beyond the 256 MB memory-side cache it is slower (n = 32, blocks of
                          2^22: 81 against 46 ms).  Never a result.  See THC_SWEEP_OK below */
} thc_params;

/* Library version (major*10000 + minor*100 + patch). */
int thc_version(void);

/* Human-readable name of a status code (static storage). */
const char* thc_strerror(int status);

/* Bytes of device workspace the calls below need for these parameters (host call, no GPU work).  The workspace
 * holds the half-transformed vectors of one group of blocks (max(2^group_log2, n * block) binary32 values, or the
 * ring of the single-launch sweep), one binary64 partial sum of squares per 8192 coordinates per worker and the
 * sweep's counters; it does not grow with d beyond those.  `ef_enabled` says whether error feedback will be used
 * (the single-launch sweep then needs a longer ring); a workspace sized with ef_enabled = 1 serves both. */
int thc_workspace_bytes(const thc_params* p, int ef_enabled, size_t* bytes_out /* host */);

/* Preliminary stage (Alg. 3: x_i = grad_i + e_i; send ||x_i||, receive the maximum; M = (t_p / sqrt(d)) * l,
 * m = -M; Sec. 5.3).  Reads every gradient once and keeps nothing but range_M.
 *   grads     host array of n device pointers, each d values of in_dtype.
 *   ef        host array of n device pointers to binary32 error-feedback buffers (read only here),
 *             or NULL when error feedback is off.
 *   range_M   device, d/block floats, written: M_k per block (m_k = -M_k).
 *   ws        device workspace of thc_workspace_bytes bytes (scratch). */
int thc_prepare_range(const thc_params* p, const void* const* grads /* host */,
                      const float* const* ef /* host or NULL */, float* range_M, void* ws, void* stream);

/* Main stage, one worker (Alg. 3: R = RHT(x), clamp, Q, SQ, Y_i, Z_i = T^-1[Y_i]; Alg. 2 worker steps; Sec. 4.1).
 *   worker_id   < n; selects the rounding stream.
 *   round       r of Alg. 3; selects the diagonal D^r and the rounding draws.  Must be < 2^32.
 *   grad        device, d values of in_dtype.
 *   ef_inout    device binary32[d] or NULL.  When given: x = grad + e is what gets compressed, and afterwards
 *               e <- x - RHT^-1(X_i) with X_i the dequantized vector (Alg. 3, error-feedback update).
 *   range_M     device, d/block floats (from thc_prepare_range, or the caller's own).
 *   packed_out  device, d*b/8 bytes, written.
 *   ws          device workspace (scratch). */
int thc_compress(const thc_params* p, uint32_t worker_id, uint64_t round, const void* grad,
                 float* ef_inout, const float* range_M, uint8_t* packed_out, void* ws, void* stream);

/* All n workers of one GPU in one sweep: what thc_prepare_range followed by thc_compress(0 .. n-1) computes, bit for
 * bit, reading every gradient (and error-feedback buffer) once: block group by block group, the transform's first
 * pass of all workers (with the norms), the range, then the last pass and the quantizer of all workers.
 *   grads       host array of n device pointers.         ef_inout    host array of n device pointers, or NULL.
 *   range_M     device, d/block floats, written.         packed_out  host array of n device pointers, written. */
int thc_compress_all(const thc_params* p, uint64_t round, const void* const* grads /* host */,
                     float* const* ef_inout /* host or NULL */, float* range_M, uint8_t* const* packed_out /* host */,
                     void* ws, void* stream);

/* Status of the last single-launch sweep (thc_params.single_launch) that used this workspace: the first 32-bit word
 * of the workspace, valid once the stream has been synchronized.  0 = fine.  1 = a workgroup waited in vain for
 * another one (workgroups were not dispatched in the order and to the XCDs the sweep counts on): every wait in the
 * kernel is bounded, nothing hangs, but that call's outputs are invalid and the caller should repeat it with
 * single_launch = 0.  Never seen on MI355X; tests and bench.py assert it is 0. */
enum { THC_SWEEP_OK = 0, THC_SWEEP_TIMEOUT = 1 };

/* Main stage, PS side (Alg. 2: Y = sum_i T[Z_i]; the PS pseudocode's lookup + aggregate steps).
 *   packed    host array of n device pointers, each d*b/8 bytes.
 *   agg_out   device, d * agg_bits/8 bytes, written.
 * Aggregating a subset of workers (partial aggregation, Sec. 6) is a call with that subset's pointers and count
 * in p->n; thc_decompress then takes the same p->n (it divides by the number of workers that were added up). */
int thc_aggregate(const thc_params* p, const uint8_t* const* packed /* host */, void* agg_out, void* stream);

/* Worker side after the PS (Alg. 2 / Alg. 3: Y_avg = Y/n; x' = m + Y_avg (M-m)/g; RHT^-1).
 *   agg   device, d * agg_bits/8 bytes.   out   device, d floats, written.   ws   device workspace. */
int thc_decompress(const thc_params* p, uint64_t round, const void* agg, const float* range_M,
                   float* out, void* ws, void* stream);

/* thc_decompress for callers that cannot allocate device memory and bring no workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same computation, bit for bit, with the
 * intermediate in a 32 MB scratch array that is part of the library's code object (one per GPU, held until the
 * process ends).  The call allocates nothing and frees nothing.  Blocks of at most 2^23 coordinates (else
 * THC_EUNSUPPORTED); d is unlimited (the vector goes through the scratch array in groups of whole blocks).
 * Every call on a GPU uses that GPU's one array: calls that overlap on the same GPU (different streams) race. */
int thc_decompress_noalloc(const thc_params* p, uint64_t round, const void* agg, const float* range_M, float* out,
                           void* stream);

/* ---- Uniform THC (Alg. 1; Sec. 4.2 "Homomorphic USQ") -----------------------------------------------
 * The simplified variant the paper generalises: 2^b uniformly spaced quantization values on the GLOBAL
 * range [m, M] = [min_i min(x_i), max_i max(x_i)] (per block), no lookup table.  `p` must carry the identity
 * table with g = 2^b - 1 (else THC_ETABLE); p->t_p is ignored.  `rotate` != 0 applies the RHT first (the
 * "with rotation" arm of the ablation in App. C): the range is then taken over the rotated vectors.
 * thc_aggregate serves unchanged (with the identity table it sums the indices).  Same pointer, stream,
 * workspace and error conventions as above. */

/* Workspace of the three calls below: min/max partials and, with rotation, the rotated vectors of all n workers
 * (n * d binary32 values, kept from thc_uniform_prepare_range to thc_uniform_compress). */
int thc_uniform_workspace_bytes(const thc_params* p, int rotate, size_t* bytes_out /* host */);

/* Preliminary stage of Alg. 1: every worker's min / max, then the global ones.
 *   range_m, range_M   device, d/block floats each, written.
 * With rotate != 0 the fully rotated vectors of all workers are left in `ws` for thc_uniform_compress. */
int thc_uniform_prepare_range(const thc_params* p, uint64_t round, const void* const* grads /* host */,
                              const float* const* ef /* host or NULL */, int rotate, float* range_m,
                              float* range_M, void* ws, void* stream);

/* Main stage of Alg. 1, worker side: X_i = USQ(x_i, m, M, b), packed.  With ef_inout:
 * e <- (grad + e) - D(X_i), through RHT^-1 when rotate != 0.  `ws` may be NULL when rotate == 0. */
int thc_uniform_compress(const thc_params* p, uint32_t worker_id, uint64_t round, const void* grad,
                         float* ef_inout, int rotate, const float* range_m, const float* range_M,
                         uint8_t* packed_out, void* ws, void* stream);

/* Alg. 1's estimate m + (1/n) X (M - m)/(2^b - 1) from the aggregated sums X (then RHT^-1 when rotate != 0). */
int thc_uniform_decompress(const thc_params* p, uint64_t round, const void* agg, int rotate,
                           const float* range_m, const float* range_M, float* out, void* ws, void* stream);

/* ---- host-side helpers (no GPU work) ------------------------------------------------------------- */

/* Introspection for tests and tools: how the Hadamard transform of these parameters is cut into passes over
 * HBM and how every pass tiles a block.  Returns the number of passes (2 to 5), or a negative status; with
 * out != NULL it also writes one record of THC_PLAN_RECORD_WORDS 32-bit words per pass (cap_records must be at
 * least the number of passes).  Record layout (unused words are 0xFFFFFFFF):
 *   [0]      0 = first pass on 8192 consecutive coordinates, 3 = first pass on 8 rows of 1024 coordinates
 *            (rows at offset bits 13..15), 1 = strided pass in place, 2 = last strided pass
 *   [1]      number of butterfly stages of the pass;  [2 .. 2+n)  their offset bits, in processing order
 *   [18..37) the tiling: L (log2 of the span the tile index runs over), log2 of the row length, number of row
 *            bits, number of tile-index bits, then the row index as two runs (length of the first run, target
 *            bit of the first run, target bit of the rest), then up to four runs of tile-index bits:
 *            4 x first tile-index bit, 4 x mask, 4 x target offset bit.
 * The offset of a coordinate inside its span is  sum_i ((tile >> first_i) & mask_i) << target_i  (tile index bits)
 * | row bits | column. */
enum { THC_PLAN_RECORD_WORDS = 40 };
int thc_describe_plan(const thc_params* p, uint32_t* out /* host, or NULL */, size_t cap_records);

/* t_p = Phi^-1(1 - p/2) (Sec. 5.1), 0 < p < 1. */
double thc_threshold(double p);

/* Optimal lookup table T_{b,g,p} of Sec. 5.2 / App. B: minimises the expected squared error of
 * stochastic quantization of a standard normal truncated to [-t_p, t_p] over tables on the (g+1)-point
 * grid.  Ties are broken towards the lexicographically smallest table.  Writes 2^b entries to
 * table_out (host) and the attained cost (in units of sigma^2) to cost_out if not NULL. */
int thc_solve_table(uint32_t b, uint32_t g, double p, uint8_t* table_out /* host */, double* cost_out /* host */);

/* The same optimum by exhaustive search: every strictly increasing table from 0 to g (the candidates App. B
 * counts; here walked as combinations of the interior values) is scored with the closed-form objective.  A cross-check of
 * thc_solve_table for small (b, g); returns THC_EUNSUPPORTED when more than 4e9 candidates would have to be
 * visited.  count_out (may be NULL) receives the number of candidates, C(g-1, 2^b-2). */
int thc_solve_table_bruteforce(uint32_t b, uint32_t g, double p, uint8_t* table_out /* host */,
                               double* cost_out /* host */, uint64_t* count_out /* host */);

#ifdef __cplusplus
}
#endif
#endif /* THC_H_ */
