"""CPU oracle for the THC data-parallel hot path (arXiv 2302.08545).

TEST INFRASTRUCTURE ONLY.  This module is a plain, slow, obviously-correct numpy
implementation of what the GPU library computes.  It may be imported only by
`tests/`, by `__graft_entry__.smoke()` and by the `cpu_baseline` leg of `bench.py`.
It shares no code, tables, constants or helpers with the HIP path and never
imports it; the product path never imports this module.

What it follows (paper passages, restated, not quoted):
  * Stochastic quantization between two bracketing values, unbiased   -- Sec. 4.1
  * Lookup table T: <2^b> -> <g+1>, granularity g                     -- Sec. 4.3
  * Worker / PS / worker steps of non-uniform THC                     -- Alg. 2
  * Randomized Hadamard transform and its inverse                     -- Sec. 5.1
  * Truncation threshold t_p and the table optimisation problem       -- Sec. 5.1, 5.2, App. B
  * Norm-based range M = (t_p / sqrt(d)) * max_i ||x_i||, m = -M      -- Sec. 5.3, Alg. 3
  * Error feedback x = grad + e,  e' = x - RHT^-1(X_i)                -- Sec. 5.1, Alg. 3
  * Stars-and-bars enumeration of candidate tables                    -- App. B, Alg. 4

Arithmetic contract.  THC is an encoding plus a randomised rounding, so the
oracle is the algorithm taken step by step in the order of Alg. 3.  Where a
floating-point value decides an integer (the table index) the decision is taken
in IEEE binary32, one rounded operation at a time, with no fused multiply-add:
that is the precision the kernels compute in, and it is what makes packed bytes
and integer sums comparable bit for bit.  Norms are accumulated in binary64.
Every convention the paper leaves open (random generator, bit order, butterfly
order, per-block scalars) is fixed in the docstring of the function that needs it.

Pins (see tests/test_oracle_*.py): Philox known-answer vectors from the Philox
publication; dense Hadamard matrices (scipy.linalg.hadamard) in binary64; H*H = B*I;
norm preservation; the paper's worked table examples (Sec. 4.3); exhaustive
enumeration of all 2^16 random half-words for the rounding probability; the
homomorphism identity; brute-force table search (Alg. 4) against the shortest-path
solver; numeric quadrature of the literal objective against the closed form.

Parity unpinned: the numerical values of the optimal tables T_{b,g,p} have no
printed reference in the paper (only this module's two independent solvers pin
each other); results that the paper shows only in figures are unpinned.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

F32 = np.float32
U32 = np.uint32
U64 = np.uint64


# --------------------------------------------------------------------------- #
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  The paper is silent on the generator; this build fixes it.
# --------------------------------------------------------------------------- #
_PHILOX_M0 = 0xD2511F53
_PHILOX_M1 = 0xCD9E8D57
_PHILOX_W0 = 0x9E3779B9
_PHILOX_W1 = 0xBB67AE85


def philox4x32_10(ctr: np.ndarray, key: Sequence[int]) -> np.ndarray:
    """Ten rounds of the Philox-4x32 bijection.

    ctr: (N, 4) uint32 counters, key: two 32-bit words.  Returns (N, 4) uint32.
    One round maps (c0, c1, c2, c3) to
        (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
    and the key is bumped by the Weyl constants between rounds.
    """
    c = np.asarray(ctr, dtype=U64).copy()
    assert c.ndim == 2 and c.shape[1] == 4
    k0 = int(key[0]) & 0xFFFFFFFF
    k1 = int(key[1]) & 0xFFFFFFFF
    mask = U64(0xFFFFFFFF)
    for _ in range(10):
        p0 = U64(_PHILOX_M0) * c[:, 0]          # 32x32 -> 64, exact in uint64
        p1 = U64(_PHILOX_M1) * c[:, 2]
        n0 = (p1 >> U64(32)) ^ c[:, 1] ^ U64(k0)
        n1 = p1 & mask
        n2 = (p0 >> U64(32)) ^ c[:, 3] ^ U64(k1)
        n3 = p0 & mask
        c = np.stack([n0, n1, n2, n3], axis=1)
        k0 = (k0 + _PHILOX_W0) & 0xFFFFFFFF
        k1 = (k1 + _PHILOX_W1) & 0xFFFFFFFF
    return c.astype(U32)


_SIGN_STREAM = 0x80000000   # fourth counter word of the sign stream


def _key_of(seed: int) -> Tuple[int, int]:
    return (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)


def rademacher_bits(seed: int, rnd: int, j0: int, count: int) -> np.ndarray:
    """Sign bits of the diagonal D^r (Sec. 5.1; one fresh diagonal per round, Alg. 3).

    Coordinate j (global index in the padded vector) takes bit (j mod 32) of word
    ((j div 32) mod 4) of Philox(counter = (q_lo, q_hi, round, 0x80000000),
    key = seed) with q = j div 128.  Bit 1 means the diagonal entry is -1.
    All workers and the decompressor share the seed, hence the diagonal.
    """
    assert 0 <= rnd < 2 ** 32
    j = np.arange(j0, j0 + count, dtype=U64)
    q = j >> U64(7)
    q_first = int(q[0]) if count else 0
    q_last = int(q[-1]) if count else -1
    qs = np.arange(q_first, q_last + 1, dtype=U64)
    ctr = np.stack([qs & U64(0xFFFFFFFF), qs >> U64(32),
                    np.full(qs.shape, rnd, dtype=U64),
                    np.full(qs.shape, _SIGN_STREAM, dtype=U64)], axis=1)
    words = philox4x32_10(ctr, _key_of(seed))              # (Q, 4)
    w = words[(q - U64(q_first)).astype(np.int64), ((j >> U64(5)) & U64(3)).astype(np.int64)]
    return ((w >> (j & U64(31)).astype(U32)) & U32(1)).astype(np.uint8)


def rademacher_signs(seed: int, rnd: int, j0: int, count: int) -> np.ndarray:
    """The diagonal of D^r as float32 +1 / -1."""
    bits = rademacher_bits(seed, rnd, j0, count)
    return np.where(bits == 1, F32(-1.0), F32(1.0)).astype(F32)


def sq_halfwords(seed: int, rnd: int, worker: int, j0: int, count: int) -> np.ndarray:
    """The 16-bit random integers that drive stochastic quantization (Sec. 4.1).

    Coordinate j of worker i in round r takes half-word (j mod 8) (low half of a
    word first, words in order) of Philox(counter = (q_lo, q_hi, r, i), key = seed)
    with q = j div 8.  Worker ids are below 2^31 so the stream never meets the sign
    stream; distinct workers draw independently (App. A asks for independence).
    """
    assert 0 <= rnd < 2 ** 32 and 0 <= worker < 2 ** 31
    j = np.arange(j0, j0 + count, dtype=U64)
    q = j >> U64(3)
    q_first = int(q[0]) if count else 0
    q_last = int(q[-1]) if count else -1
    qs = np.arange(q_first, q_last + 1, dtype=U64)
    ctr = np.stack([qs & U64(0xFFFFFFFF), qs >> U64(32),
                    np.full(qs.shape, rnd, dtype=U64),
                    np.full(qs.shape, worker, dtype=U64)], axis=1)
    words = philox4x32_10(ctr, _key_of(seed))
    i = (j & U64(7)).astype(np.int64)
    w = words[(q - U64(q_first)).astype(np.int64), i >> 1]
    return ((w >> (U32(16) * (i & 1).astype(U32))) & U32(0xFFFF)).astype(U32)


def sq_uniform_from_halfword(h: np.ndarray) -> np.ndarray:
    """u = (h + 1/2) / 2^16: a uniform on the centred 2^16-point grid of (0, 1); exact in binary32."""
    return ((h.astype(F32) + F32(0.5)) * F32(1.0 / 65536.0)).astype(F32)


# --------------------------------------------------------------------------- #
# Parameters
# --------------------------------------------------------------------------- #
@dataclass
class Params:
    """The problem statement of Alg. 3: d, n, b, g, table, seed, p (as t_p)."""
    d: int                  # padded coordinate count, a multiple of `block`
    block: int              # B: the RHT is applied to each block of B coordinates (power of two)
    n: int                  # workers
    b: int                  # index bits per coordinate
    g: int                  # granularity
    t_p: float              # Phi^-1(1 - p/2), stored as binary32
    seed: int               # shared 64-bit seed
    table: Sequence[int]    # T[0..2^b-1], 0 = T[0] < ... < T[2^b-1] = g
    agg_bits: int = 8       # width of one aggregated value (1..16 bits)
    order: int = 0          # butterfly stage order, see stage_order()
    F: np.ndarray = field(init=False, repr=False)

    def __post_init__(self):
        self.t_p = float(F32(self.t_p))
        T = [int(v) for v in self.table]
        assert len(T) == 2 ** self.b
        assert T[0] == 0 and T[-1] == self.g and all(T[i] < T[i + 1] for i in range(len(T) - 1)), \
            "homomorphism precondition of Sec. 4.3: 0 = T[0] < ... < T[2^b-1] = g"
        assert self.block & (self.block - 1) == 0 and self.d % self.block == 0
        assert 1 <= self.b <= 8 and 1 <= self.agg_bits <= 16
        assert self.g * self.n < 2 ** self.agg_bits, "aggregated sums must fit (Sec. 8 setup: g*n <= 255 at 8 bits)"
        self.table = T
        # F[k] = largest index z with T[z] <= k, for every grid cell k in 0..g
        self.F = np.array([max(z for z in range(len(T)) if T[z] <= k) for k in range(self.g + 1)],
                          dtype=np.int64)

    @property
    def K(self) -> int:
        return self.d // self.block


# --------------------------------------------------------------------------- #
# Hadamard transform (Sec. 5.1).  Natural (Sylvester) order, H[i][j] = (-1)^popcount(i & j),
# evaluated by radix-2 butterflies in ascending stride order.  The stride order is
# part of the numeric contract: binary32 additions are not associative.
# --------------------------------------------------------------------------- #
def fwht_loops(x: Sequence[float]) -> np.ndarray:
    """Literal triple loop, binary32, for tiny inputs: stride h = 1, 2, 4, ...;
    every pair (j, j+h) with bit h of j clear becomes (a + b, a - b)."""
    y = np.array(x, dtype=F32)
    B = y.size
    h = 1
    while h < B:
        for j in range(B):
            if j & h == 0:
                a, b = y[j], y[j + h]
                y[j], y[j + h] = F32(a + b), F32(a - b)
        h *= 2
    return y


def stage_order(B: int, order: int = 0) -> List[int]:
    """The bit positions of the butterfly stages, in processing order (a stage on bit k pairs coordinates
    whose offsets in the block differ by 2^k).  order 0: ascending, 0, 1, ..., log2(B)-1.  order 1 ("split"),
    for B >= 2^16: 0..9, 13, 14, 15, then 10, 11, 12, 16, ..., log2(B)-1; ascending for smaller blocks.
    Any order computes H x exactly in exact arithmetic; binary32 roundings depend on it."""
    L = B.bit_length() - 1
    if order == 1 and L >= 16:
        return list(range(10)) + [13, 14, 15, 10, 11, 12] + list(range(16, L))
    return list(range(L))


def fwht_f32(x: np.ndarray, bits: Optional[Sequence[int]] = None) -> np.ndarray:
    """Same butterflies as `fwht_loops`, vectorised, along the last axis (binary32); `bits` lists the
    stages (bit positions) in processing order, ascending by default."""
    y = np.array(x, dtype=F32, copy=True)
    B = y.shape[-1]
    assert B & (B - 1) == 0
    L = B.bit_length() - 1
    if bits is None:
        bits = range(L)
    assert sorted(bits) == list(range(L))
    lead = y.shape[:-1]
    for k in bits:
        h = 1 << k
        v = y.reshape(lead + (B // (2 * h), 2, h))
        a = v[..., 0, :].copy()
        b = v[..., 1, :].copy()
        v[..., 0, :] = a + b
        v[..., 1, :] = a - b
    return y


def rht_scale(B: int) -> np.float32:
    """c = 1/sqrt(B), computed in binary64 and rounded once (a power of two for even log2 B)."""
    return F32(1.0 / math.sqrt(float(B)))


def rht_blocks(x: np.ndarray, signs: np.ndarray, B: int, order: int = 0) -> np.ndarray:
    """RHT(x) = (1/sqrt(B)) H D x on every block of B coordinates (Sec. 5.1)."""
    v = (x.astype(F32) * signs).reshape(-1, B)
    return (fwht_f32(v, stage_order(B, order)) * rht_scale(B)).astype(F32).reshape(-1)


def irht_blocks(v: np.ndarray, signs: np.ndarray, B: int, order: int = 0) -> np.ndarray:
    """RHT^-1(v) = (1/sqrt(B)) D H v on every block (Sec. 5.1)."""
    h = fwht_f32(v.astype(F32).reshape(-1, B), stage_order(B, order)).reshape(-1)
    return ((h * rht_scale(B)).astype(F32) * signs).astype(F32)


# --------------------------------------------------------------------------- #
# Preliminary stage: the shared range (Sec. 5.3; Alg. 3, norm exchange and M)
# --------------------------------------------------------------------------- #
def ef_input(grad: np.ndarray, ef: Optional[np.ndarray]) -> np.ndarray:
    """x = grad + e (Alg. 3).  bfloat16 gradients arrive already widened (exact)."""
    x = np.asarray(grad, dtype=F32)
    if ef is not None:
        x = (x + np.asarray(ef, dtype=F32)).astype(F32)
    return x


def prepare_range(P: Params, grads: Sequence[np.ndarray],
                  efs: Optional[Sequence[np.ndarray]] = None) -> np.ndarray:
    """M_k for every block k: M = t_p * l / sqrt(B) with l the largest worker norm of
    that block (unsquared L2 norm, as in Alg. 3), m = -M.

    Sum of squares in binary64 (each square of a binary32 number is exact there);
    M_k = float32( float64(t_p) * sqrt(max_i s_i) / sqrt(float64(B)) ).
    """
    smax = np.zeros(P.K, dtype=np.float64)
    for i in range(P.n):
        x = ef_input(grads[i], None if efs is None else efs[i]).astype(np.float64)
        s = np.array([np.sum(blk * blk) for blk in x.reshape(P.K, P.block)], dtype=np.float64)
        smax = np.maximum(smax, s)
    M = (np.float64(P.t_p) * np.sqrt(smax)) / np.sqrt(np.float64(P.block))
    return M.astype(F32)


# --------------------------------------------------------------------------- #
# Bit packing (paper silent): a stream of w-bit fields, field j occupying bits [j*w, j*w + w) of the
# stream, the stream's bit k being bit (k mod 8) of byte (k div 8) -- least-significant bits first.
# Used for the index stream (w = b) and for the aggregated stream (w = agg_bits).
# --------------------------------------------------------------------------- #
def pack_fields(values: np.ndarray, w: int) -> np.ndarray:
    assert 1 <= w <= 16
    v = np.asarray(values, dtype=np.uint32)
    assert (v.size * w) % 8 == 0 and int(v.max(initial=0)) < (1 << w)
    bits = ((v[:, None] >> np.arange(w, dtype=np.uint32)[None, :]) & 1).astype(np.uint8)   # field-major, LSB first
    return np.packbits(bits.reshape(-1), bitorder="little")


def unpack_fields(packed: np.ndarray, w: int) -> np.ndarray:
    assert 1 <= w <= 16
    bits = np.unpackbits(np.asarray(packed, dtype=np.uint8), bitorder="little").reshape(-1, w).astype(np.uint32)
    return (bits << np.arange(w, dtype=np.uint32)[None, :]).sum(axis=1).astype(np.uint32)


def pack_indices(z: np.ndarray, b: int) -> np.ndarray:
    return pack_fields(z, b)


def unpack_indices(packed: np.ndarray, b: int) -> np.ndarray:
    return unpack_fields(packed, b).astype(np.uint8)


# --------------------------------------------------------------------------- #
# Main stage, worker side (Alg. 3: clamp, SQ, Y, Z) and error feedback
# --------------------------------------------------------------------------- #
def block_scalars(P: Params, range_M: np.ndarray, range_m: Optional[np.ndarray] = None):
    """Per-block constants derived from the range [m, M] (m = -M unless given), each a binary64 quotient
    rounded once to binary32, with the width M - m taken in binary64:
    scale = g/(M-m),  step_g = (M-m)/g,  step_n = (M-m)/(g n).
    The grid position of Alg. 2 needs g/(M-m) as a binary32 number.  Where that quotient is not a finite binary32
    value -- M = m (the all-zero block), or a width so small that it overflows -- the range is empty: scale 0, so
    that every coordinate maps to index 0 (and decodes to m)."""
    M64 = range_M.astype(np.float64)
    m64 = -M64 if range_m is None else range_m.astype(np.float64)
    W64 = M64 - m64
    with np.errstate(divide="ignore", invalid="ignore", over="ignore"):
        scale = (np.float64(P.g) / W64).astype(F32)
    scale = np.where(np.isfinite(scale), scale, F32(0.0)).astype(F32)
    step_g = (W64 / np.float64(P.g)).astype(F32)
    step_n = (W64 / np.float64(P.g * P.n)).astype(F32)
    return scale, step_g, step_n


def _lower(range_M: np.ndarray, range_m: Optional[np.ndarray]) -> np.ndarray:
    return (-range_M.astype(F32)) if range_m is None else range_m.astype(F32)


def quantize_rotated(P: Params, R: np.ndarray, range_M: np.ndarray, h16: np.ndarray,
                     range_m: Optional[np.ndarray] = None) -> np.ndarray:
    """Clamp + stochastic quantization onto the table's values + inverse table lookup.

    R: (rotated) coordinates (float32, length d); h16: the 16-bit random integers.
    Per coordinate, all in binary32:
        x' = min(max(R, m), M)                       truncation (Alg. 3)
        y  = (x' - m) * scale          in [0, g]     position on the (g+1)-point grid
        k  = min(floor(y), g);  z0 = F[k]            largest index whose table value is <= y
        top index: stays.  Otherwise lo = T[z0], wd = T[z0+1] - lo, t = y - lo and the
        value goes up to z0+1 exactly when u * wd < t, with u = (h16 + 1/2) / 2^16.
    So P(up) = t/wd up to 2^-17: the quantization of Sec. 4.1, unbiased.
    Returns indices z in <2^b> (Alg. 2's Z = T^-1[Y]).
    """
    B = P.block
    scale, _, _ = block_scalars(P, range_M, range_m)
    M = np.repeat(range_M.astype(F32), B)
    m = np.repeat(_lower(range_M, range_m), B)
    sc = np.repeat(scale, B)
    xc = np.minimum(np.maximum(R.astype(F32), m), M)
    y = ((xc - m).astype(F32) * sc).astype(F32)
    k = np.minimum(np.floor(y).astype(np.int64), P.g)
    z0 = P.F[k]
    T = np.array(list(P.table) + [P.table[-1]], dtype=np.int64)   # sentinel for the top index
    lo = T[z0]
    wd = T[z0 + 1] - lo
    t = (y - lo.astype(F32)).astype(F32)
    u = sq_uniform_from_halfword(h16)
    up = ((u * wd.astype(F32)).astype(F32) < t) & (z0 < (2 ** P.b - 1))
    return (z0 + up.astype(np.int64)).astype(np.uint8)


def dequantize_indices(P: Params, z: np.ndarray, range_M: np.ndarray,
                       range_m: Optional[np.ndarray] = None) -> np.ndarray:
    """X = m + T[z] (M - m)/g  (Sec. 4.3, Alg. 2), binary32: float(T[z]) * step_g, then + m."""
    _, step_g, _ = block_scalars(P, range_M, range_m)
    Tz = np.array(P.table, dtype=np.int64)[z.astype(np.int64)].astype(F32)
    sg = np.repeat(step_g, P.block)
    m = np.repeat(_lower(range_M, range_m), P.block)
    return ((Tz * sg).astype(F32) + m).astype(F32)


def compress(P: Params, worker: int, rnd: int, grad: np.ndarray, ef: Optional[np.ndarray],
             range_M: np.ndarray, j0: int = 0) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """One worker's round (Alg. 3): x = grad + e, R = RHT(x), clamp, SQ, index, pack.
    Returns (packed bytes, new error-feedback buffer or None).

    j0 is the global index of the first coordinate (for sampling blocks of a long vector).
    Error feedback, literally: e' = x - RHT^-1(X) with X the dequantized vector.
    """
    d = grad.size
    assert d == P.d
    x = ef_input(grad, ef)
    signs = rademacher_signs(P.seed, rnd, j0, d)
    R = rht_blocks(x, signs, P.block, P.order)
    h16 = sq_halfwords(P.seed, rnd, worker, j0, d)
    z = quantize_rotated(P, R, range_M, h16)
    packed = pack_indices(z, P.b)
    new_ef = None
    if ef is not None:
        X = dequantize_indices(P, z, range_M)
        new_ef = (x - irht_blocks(X, signs, P.block, P.order)).astype(F32)
    return packed, new_ef


# --------------------------------------------------------------------------- #
# Main stage, PS side (Alg. 2: Y = sum_i T[Z_i]) and worker-side decompression
# --------------------------------------------------------------------------- #
def aggregate(P: Params, packed: Sequence[np.ndarray]) -> np.ndarray:
    """Y[j] = sum over workers of T[Z_i[j]], exact integers (uint8 if they fit a byte, else uint16)."""
    T = np.array(P.table, dtype=np.int64)
    Y = np.zeros(P.d, dtype=np.int64)
    for pk in packed:
        Y += T[unpack_indices(pk, P.b).astype(np.int64)]
    assert Y.max(initial=0) < 2 ** P.agg_bits
    return Y.astype(np.uint8 if P.agg_bits <= 8 else np.uint16)


def aggregate_stream(P: Params, Y: np.ndarray) -> np.ndarray:
    """The aggregated sums as the byte stream a PS would send: agg_bits per coordinate (Sec. 8.4 notes that
    ceil(log2(g n + 1)) bits suffice)."""
    return pack_fields(Y, P.agg_bits)


def decompress(P: Params, rnd: int, Y: np.ndarray, range_M: np.ndarray, j0: int = 0) -> np.ndarray:
    """Estimate of the average gradient: m + (Y/n)(M-m)/g, then RHT^-1 (Alg. 2 / Alg. 3).
    binary32: v = float(Y) * step_n + m with step_n = (M-m)/(g n), m = -M; out = (H v) * c * sign."""
    _, _, step_n = block_scalars(P, range_M)
    sn = np.repeat(step_n, P.block)
    M = np.repeat(range_M.astype(F32), P.block)
    v = ((Y.astype(F32) * sn).astype(F32) + (-M)).astype(F32)
    signs = rademacher_signs(P.seed, rnd, j0, P.d)
    return irht_blocks(v, signs, P.block, P.order)


# --------------------------------------------------------------------------- #
# Uniform THC (Alg. 1): identity table with g = 2^b - 1, range = global minimum and maximum of what is
# quantized (the gradients themselves, or their RHT when rotation is switched on -- the ablation of App. C).
# --------------------------------------------------------------------------- #
def uniform_values(P: Params, rnd: int, grad: np.ndarray, ef: Optional[np.ndarray], rotate: bool,
                   j0: int = 0) -> np.ndarray:
    """What a worker quantizes: x = grad + e, rotated block-wise when `rotate`.  j0 is the global index of the
    first coordinate (as in `compress`)."""
    x = ef_input(grad, ef)
    if rotate:
        x = rht_blocks(x, rademacher_signs(P.seed, rnd, j0, P.d), P.block, P.order)
    return x


def uniform_range(P: Params, rnd: int, grads: Sequence[np.ndarray], efs: Optional[Sequence[np.ndarray]],
                  rotate: bool, j0: int = 0) -> Tuple[np.ndarray, np.ndarray]:
    """Preliminary stage of Alg. 1: (m_k, M_k) = (min, max) over all workers of block k."""
    lo = np.full(P.K, np.inf, dtype=F32)
    hi = np.full(P.K, -np.inf, dtype=F32)
    for i in range(P.n):
        v = uniform_values(P, rnd, grads[i], None if efs is None else efs[i], rotate, j0).reshape(P.K, P.block)
        lo = np.minimum(lo, v.min(axis=1))
        hi = np.maximum(hi, v.max(axis=1))
    return lo, hi


def uniform_compress(P: Params, worker: int, rnd: int, grad: np.ndarray, ef: Optional[np.ndarray],
                     range_m: np.ndarray, range_M: np.ndarray, rotate: bool, j0: int = 0):
    """Main stage of Alg. 1, worker side: X_i = USQ(x_i, m, M, b), packed; with error feedback
    e' = x - D(X_i) (through RHT^-1 when rotated).  P must carry the identity table (g = 2^b - 1)."""
    assert list(P.table) == list(range(2 ** P.b)) and P.g == 2 ** P.b - 1
    x = ef_input(grad, ef)
    v = uniform_values(P, rnd, grad, ef, rotate, j0)
    z = quantize_rotated(P, v, range_M, sq_halfwords(P.seed, rnd, worker, j0, P.d), range_m)
    new_ef = None
    if ef is not None:
        X = dequantize_indices(P, z, range_M, range_m)
        if rotate:
            X = irht_blocks(X, rademacher_signs(P.seed, rnd, j0, P.d), P.block, P.order)
        new_ef = (x - X).astype(F32)
    return pack_indices(z, P.b), new_ef


def uniform_decompress(P: Params, rnd: int, Y: np.ndarray, range_m: np.ndarray, range_M: np.ndarray,
                       rotate: bool, j0: int = 0) -> np.ndarray:
    """Alg. 1's estimate m + (1/n) X (M-m)/(2^b-1) (then RHT^-1 when rotated); X is the integer sum."""
    _, _, step_n = block_scalars(P, range_M, range_m)
    v = ((Y.astype(F32) * np.repeat(step_n, P.block)).astype(F32) + np.repeat(range_m.astype(F32), P.block)).astype(F32)
    if rotate:
        v = irht_blocks(v, rademacher_signs(P.seed, rnd, j0, P.d), P.block, P.order)
    return v


def thc_round(P: Params, rnd: int, grads: Sequence[np.ndarray],
              efs: Optional[List[np.ndarray]] = None):
    """One full round for n workers held in one process.  Returns
    (range_M, [packed_i], Y, average estimate, [new ef_i] or None)."""
    M = prepare_range(P, grads, efs)
    packed, new_efs = [], []
    for i in range(P.n):
        pk, ne = compress(P, i, rnd, grads[i], None if efs is None else efs[i], M)
        packed.append(pk)
        new_efs.append(ne)
    Y = aggregate(P, packed)
    out = decompress(P, rnd, Y, M)
    return M, packed, Y, out, (new_efs if efs is not None else None)


def nmse(x: np.ndarray, xhat: np.ndarray) -> float:
    """||x - xhat||^2 / ||x||^2 (Sec. 2.1)."""
    x = x.astype(np.float64)
    return float(np.sum((x - xhat.astype(np.float64)) ** 2) / np.sum(x * x))


# --------------------------------------------------------------------------- #
# Offline: truncation threshold and the optimal lookup table (Sec. 5.2, App. B)
# --------------------------------------------------------------------------- #
def t_p_of(p: float) -> float:
    """t_p = Phi^-1(1 - p/2)."""
    from scipy.special import ndtri
    return float(-ndtri(p / 2.0))       # = Phi^-1(1 - p/2) by symmetry, without the cancellation in 1 - p/2


def _phi(a):
    return math.exp(-0.5 * a * a) / math.sqrt(2.0 * math.pi)


def _Phi(a):
    return 0.5 * math.erfc(-a / math.sqrt(2.0))


def pair_cost(q0: float, q1: float) -> float:
    """Expected squared error contributed by values between adjacent quantization values
    q0 < q1 of a standard normal: with SQ the conditional variance at a is (a-q0)(q1-a), so
    the cost is  integral_{q0}^{q1} (a - q0)(q1 - a) phi(a) da, in closed form through
    int phi = dPhi,  int a phi = -dphi,  int a^2 phi = dPhi - d(a phi)."""
    dPhi = _Phi(q1) - _Phi(q0)
    dphi = _phi(q1) - _phi(q0)
    daphi = q1 * _phi(q1) - q0 * _phi(q0)
    i0, i1, i2 = dPhi, -dphi, dPhi - daphi
    return -i2 + (q0 + q1) * i1 - q0 * q1 * i0


def table_cost(table: Sequence[int], g: int, t_p: float) -> float:
    """Objective of Sec. 5.2 for a given table, with P fixed to SQ between neighbours."""
    q = [-t_p + v * 2.0 * t_p / g for v in table]
    return sum(pair_cost(q[i], q[i + 1]) for i in range(len(q) - 1))


def solve_table(b: int, g: int, p: float, rel_tie: float = 1e-12) -> List[int]:
    """Optimal T_{b,g,p}.  The objective is a sum over consecutive table values, so the optimum
    is a cheapest path with 2^b - 1 edges from grid point 0 to grid point g.  Ties (a table and
    its mirror for even g) are broken towards the lexicographically smallest table."""
    L = 2 ** b - 1
    assert g >= L
    tp = t_p_of(p)
    qv = [-tp + v * 2.0 * tp / g for v in range(g + 1)]
    w = [[pair_cost(qv[i], qv[j]) if j > i else math.inf for j in range(g + 1)] for i in range(g + 1)]
    INF = math.inf
    # best[e][v] = cheapest cost from v to g using exactly e edges
    best = [[INF] * (g + 1) for _ in range(L + 1)]
    best[0][g] = 0.0
    for e in range(1, L + 1):
        for v in range(g + 1):
            best[e][v] = min((w[v][u] + best[e - 1][u] for u in range(v + 1, g + 1)), default=INF)
    opt = best[L][0]
    tol = abs(opt) * rel_tie
    table, v, spent = [0], 0, 0.0
    for e in range(L, 0, -1):
        for u in range(v + 1, g + 1):
            if spent + w[v][u] + best[e - 1][u] <= opt + tol:
                spent += w[v][u]
                table.append(u)
                v = u
                break
        else:
            raise AssertionError("reconstruction failed")
    return table


def stars_and_bars(n: int, k: int):
    """All ways to put n identical balls into k bins (App. B, Alg. 4): start with every ball in
    bin 0; repeatedly take the first non-empty bin a, move one ball to bin a+1 and the rest of
    bin a back to bin 0; stop after C(n+k-1, k-1) arrangements."""
    B = [0] * k
    B[0] = n
    total = math.comb(n + k - 1, k - 1)
    yield list(B)
    for _ in range(1, total):
        a = next(i for i in range(k) if B[i] > 0)
        B[a + 1] += 1
        s = B[a] - 1
        B[a] = 0
        B[0] = s
        yield list(B)


def enumerate_tables(b: int, g: int):
    """Every strictly increasing table with T[0] = 0, T[2^b-1] = g: the 2^b - 1 gaps are all >= 1
    and sum to g, i.e. g - (2^b - 1) spare units thrown into 2^b - 1 bins."""
    L = 2 ** b - 1
    for bins in stars_and_bars(g - L, L):
        t = [0]
        for extra in bins:
            t.append(t[-1] + 1 + extra)
        yield t
