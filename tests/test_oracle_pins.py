"""Pins for the CPU oracle: everything here checks `oracle/` against something other than
itself -- values the paper prints, published known-answer vectors, library routines,
closed forms, brute force on tiny inputs, exhaustive enumeration, invariants.  No GPU."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.integrate
import scipy.linalg
import scipy.stats

from oracle import thc_oracle as o

F32 = np.float32
TP32 = o.t_p_of(1 / 32)
T430 = [0, 3, 5, 7, 9, 11, 13, 14, 15, 17, 19, 21, 23, 25, 27, 30]


def _params(d=4096, block=1024, n=4, b=4, g=30, table=None, agg_bits=8, seed=0x5448435F53454544):
    return o.Params(d=d, block=block, n=n, b=b, g=g, t_p=TP32, seed=seed,
                    table=table if table is not None else T430, agg_bits=agg_bits)


# ------------------------------------------------------------------ Philox
def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r if x != "->"]
        out = o.philox4x32_10(np.array([v[0:4]], dtype=np.uint32), v[4:6])[0]
        assert [int(x) for x in out] == v[6:10]


def test_philox_is_a_bijection_per_key_on_a_sample():
    # distinct counters give distinct outputs (Philox is a permutation of the counter space)
    ctr = np.zeros((4096, 4), dtype=np.uint32)
    ctr[:, 0] = np.arange(4096)
    out = o.philox4x32_10(ctr, (7, 9))
    assert len({tuple(r) for r in out.tolist()}) == 4096


def test_halfword_stream_uniformity():
    h = o.sq_halfwords(seed=1234567, rnd=3, worker=2, j0=0, count=1 << 20).astype(np.int64)
    assert h.min() >= 0 and h.max() < 65536
    # mean of a uniform on 0..65535 is 32767.5 with sd 18918/sqrt(N)
    assert abs(h.mean() - 32767.5) < 5 * 18918.0 / math.sqrt(h.size)
    counts = np.bincount(h >> 8, minlength=256)
    chi2 = ((counts - h.size / 256) ** 2 / (h.size / 256)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 255)
    # low bits too
    counts = np.bincount(h & 255, minlength=256)
    chi2 = ((counts - h.size / 256) ** 2 / (h.size / 256)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 255)


def test_stream_windows_are_slices_and_streams_are_distinct():
    seed = 0xDEADBEEFCAFE
    full_h = o.sq_halfwords(seed, 5, 1, 0, 5000)
    full_s = o.rademacher_bits(seed, 5, 0, 5000)
    for j0, cnt in [(0, 17), (3, 100), (127, 130), (1024, 999), (4093, 907)]:
        assert np.array_equal(o.sq_halfwords(seed, 5, 1, j0, cnt), full_h[j0:j0 + cnt])
        assert np.array_equal(o.rademacher_bits(seed, 5, j0, cnt), full_s[j0:j0 + cnt])
    assert not np.array_equal(o.sq_halfwords(seed, 5, 2, 0, 5000), full_h)      # other worker
    assert not np.array_equal(o.sq_halfwords(seed, 6, 1, 0, 5000), full_h)      # other round
    assert not np.array_equal(o.rademacher_bits(seed, 6, 0, 5000), full_s)      # D^r changes per round
    assert not np.array_equal(o.rademacher_bits(seed + 1, 5, 0, 5000), full_s)


def test_stream_layout_against_direct_philox_call():
    # coordinate j = 8q + i uses half (i&1) of word (i>>1) of Philox((q, 0, round, worker))
    seed, rnd, worker = 0x0123456789ABCDEF, 9, 4
    key = (seed & 0xFFFFFFFF, seed >> 32)
    w = o.philox4x32_10(np.array([[5, 0, rnd, worker]], dtype=np.uint32), key)[0]
    h = o.sq_halfwords(seed, rnd, worker, 40, 8)
    expect = []
    for word in w:
        expect += [int(word) & 0xFFFF, int(word) >> 16]
    assert h.tolist() == expect
    # sign bit of coordinate j = 128q + 32w + t is bit t of word w of Philox((q, 0, round, 0x80000000))
    w = o.philox4x32_10(np.array([[2, 0, rnd, 0x80000000]], dtype=np.uint32), key)[0]
    bits = o.rademacher_bits(seed, rnd, 256, 128)
    expect = [(int(w[t // 32]) >> (t % 32)) & 1 for t in range(128)]
    assert bits.tolist() == expect
    s = o.rademacher_signs(seed, rnd, 256, 128)
    assert np.array_equal(s, np.where(np.array(expect) == 1, -1.0, 1.0).astype(F32))


def test_rademacher_balance():
    bits = o.rademacher_bits(42, 0, 0, 1 << 20).astype(np.int64)
    assert abs(bits.mean() - 0.5) < 5 * 0.5 / math.sqrt(bits.size)
    # no obvious lag-1 correlation
    corr = np.mean((2 * bits[1:] - 1) * (2 * bits[:-1] - 1))
    assert abs(corr) < 5 / math.sqrt(bits.size)


# ------------------------------------------------------------------ Hadamard / RHT
@pytest.mark.parametrize("B", [2, 4, 8, 64, 256, 1024])
def test_fwht_equals_dense_hadamard(B):
    rng = np.random.default_rng(B)
    x = rng.standard_normal(B).astype(F32)
    ref = scipy.linalg.hadamard(B).astype(np.float64) @ x.astype(np.float64)
    got = o.fwht_f32(x).astype(np.float64)
    assert np.linalg.norm(got - ref) <= 1e-6 * np.linalg.norm(ref)
    if B <= 64:
        assert np.array_equal(o.fwht_loops(x), o.fwht_f32(x))


def test_fwht_loops_equals_vectorised_exactly():
    rng = np.random.default_rng(7)
    for B in (2, 16, 128, 512):
        x = (rng.standard_normal(B) * 10 ** rng.uniform(-4, 2)).astype(F32)
        assert np.array_equal(o.fwht_loops(x), o.fwht_f32(x))


def test_fwht_unit_vectors_give_hadamard_columns_exactly():
    B = 64
    H = scipy.linalg.hadamard(B)
    for j in (0, 1, 2, 5, 31, 63):
        e = np.zeros(B, dtype=F32)
        e[j] = 1
        assert np.array_equal(o.fwht_f32(e), H[:, j].astype(F32))     # entries are (-1)^popcount(i&j)
    i, j = 0b101101, 0b011100
    assert H[i, j] == (-1) ** bin(i & j).count("1")


def test_fwht_textbook_size_two_and_involution():
    assert o.fwht_f32(np.array([3.0, 5.0], dtype=F32)).tolist() == [8.0, -2.0]
    # H H = B I: exact on small integers (all intermediate values are exactly representable)
    rng = np.random.default_rng(0)
    x = rng.integers(-50, 50, size=1024).astype(F32)
    assert np.array_equal(o.fwht_f32(o.fwht_f32(x)), x * F32(1024))


def test_fwht_any_stage_order_is_the_same_transform():
    # the order of the butterfly stages only moves roundings: every order equals the dense product, and is exact on
    # small integers
    rng = np.random.default_rng(1)
    B = 256
    H = scipy.linalg.hadamard(B).astype(np.float64)
    x = rng.standard_normal(B).astype(F32)
    xi = rng.integers(-20, 20, size=B).astype(F32)
    for _ in range(5):
        bits = rng.permutation(8).tolist()
        got = o.fwht_f32(x, bits).astype(np.float64)
        assert np.linalg.norm(got - H @ x) <= 1e-6 * np.linalg.norm(H @ x)
        assert np.array_equal(o.fwht_f32(xi, bits), (H @ xi).astype(F32))
    assert np.array_equal(o.fwht_f32(x, list(range(8))), o.fwht_f32(x))
    with pytest.raises(AssertionError):
        o.fwht_f32(x, [0, 1, 2, 3, 4, 5, 6, 6])                   # every bit exactly once


def test_stage_order_conventions():
    assert o.stage_order(1 << 20, 0) == list(range(20))
    assert o.stage_order(1 << 20, 1) == list(range(10)) + [13, 14, 15, 10, 11, 12, 16, 17, 18, 19]
    assert o.stage_order(1 << 16, 1) == list(range(10)) + [13, 14, 15, 10, 11, 12]
    assert o.stage_order(1 << 15, 1) == list(range(15))           # below 2^16 the split order is the ascending one
    for L in (10, 13, 16, 22, 25, 27):
        assert sorted(o.stage_order(1 << L, 1)) == list(range(L))
    # the two orders differ in roundings only
    rng = np.random.default_rng(3)
    x = rng.standard_normal(1 << 16).astype(F32)
    s = o.rademacher_signs(5, 0, 0, 1 << 16)
    a, b = o.rht_blocks(x, s, 1 << 16, 0), o.rht_blocks(x, s, 1 << 16, 1)
    assert not np.array_equal(a, b)
    assert np.linalg.norm(a.astype(np.float64) - b) <= 1e-6 * np.linalg.norm(a)


def test_fwht_blocks_along_last_axis():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((5, 256)).astype(F32)
    got = o.fwht_f32(x)
    for r in range(5):
        assert np.array_equal(got[r], o.fwht_f32(x[r]))


@pytest.mark.parametrize("B", [256, 1024, 4096])
def test_rht_preserves_norm_and_inverts(B):
    rng = np.random.default_rng(11)
    d = 4 * B
    x = rng.standard_normal(d).astype(F32)
    s = o.rademacher_signs(99, 1, 0, d)
    R = o.rht_blocks(x, s, B)
    for k in range(4):
        nb = np.linalg.norm(x[k * B:(k + 1) * B].astype(np.float64))
        assert abs(np.linalg.norm(R[k * B:(k + 1) * B].astype(np.float64)) - nb) < 1e-5 * nb
    back = o.irht_blocks(R, s, B)
    assert np.linalg.norm(back.astype(np.float64) - x) <= 1e-6 * np.linalg.norm(x)


def test_rht_matches_dense_definition():
    # (1/sqrt(d)) H D x with a dense H and an explicit diagonal, in binary64
    B = 512
    rng = np.random.default_rng(5)
    x = rng.standard_normal(B).astype(F32)
    s = o.rademacher_signs(17, 2, 0, B)
    H = scipy.linalg.hadamard(B).astype(np.float64)
    ref = H @ (np.diag(s.astype(np.float64)) @ x.astype(np.float64)) / math.sqrt(B)
    got = o.rht_blocks(x, s, B).astype(np.float64)
    assert np.linalg.norm(got - ref) <= 1e-6 * np.linalg.norm(ref)
    inv_ref = np.diag(s.astype(np.float64)) @ (H @ x.astype(np.float64)) / math.sqrt(B)
    got = o.irht_blocks(x, s, B).astype(np.float64)
    assert np.linalg.norm(got - inv_ref) <= 1e-6 * np.linalg.norm(inv_ref)


def test_rht_output_looks_gaussian_with_variance_norm2_over_d():
    # Sec. 5.1: rotated coordinates approach N(0, ||x||^2/d); about a p fraction falls outside +-t_p sigma
    B = 1 << 16
    rng = np.random.default_rng(2)
    x = rng.laplace(size=B).astype(F32) * F32(1e-3)          # far from Gaussian before rotation
    s = o.rademacher_signs(1, 0, 0, B)
    R = o.rht_blocks(x, s, B).astype(np.float64)
    sigma = np.linalg.norm(x.astype(np.float64)) / math.sqrt(B)
    assert abs(R.std() - sigma) < 1e-3 * sigma * 10
    frac = np.mean(np.abs(R) > TP32 * sigma)
    assert abs(frac - 1 / 32) < 5 * math.sqrt((1 / 32) / B)
    assert abs(scipy.stats.kurtosis(R)) < 0.1                   # Laplace input has excess kurtosis 3


# ------------------------------------------------------------------ range
def test_range_constant_vector_closed_form():
    P = _params(d=2048, block=1024, n=2)
    g0 = np.full(2048, 0.5, dtype=F32)
    g1 = np.full(2048, -0.25, dtype=F32)
    M = o.prepare_range(P, [g0, g1])
    # ||g0 block|| = 0.5*sqrt(1024) = 16 -> M = t_p*16/32
    assert M.dtype == F32 and M.shape == (2,)
    assert np.array_equal(M, np.full(2, F32(np.float64(F32(TP32)) * 16.0 / 32.0)))


def test_range_uses_max_worker_norm_per_block_and_ef():
    P = _params(d=2048, block=1024, n=3)
    rng = np.random.default_rng(1)
    grads = [rng.standard_normal(2048).astype(F32) * F32(sc) for sc in (1.0, 3.0, 2.0)]
    grads[0][1024:] *= F32(10)                                   # block 1: worker 0 dominates
    M = o.prepare_range(P, grads)
    n0 = [np.linalg.norm(g[:1024].astype(np.float64)) for g in grads]
    n1 = [np.linalg.norm(g[1024:].astype(np.float64)) for g in grads]
    assert np.argmax(n0) == 1 and np.argmax(n1) == 0
    assert M[0] == pytest.approx(TP32 * max(n0) / 32, rel=1e-6)
    assert M[1] == pytest.approx(TP32 * max(n1) / 32, rel=1e-6)
    efs = [np.full(2048, 100.0, dtype=F32) for _ in range(3)]
    M2 = o.prepare_range(P, grads, efs)                          # x = grad + e enters the norm
    assert M2[0] == pytest.approx(
        TP32 * max(np.linalg.norm((g[:1024] + F32(100)).astype(np.float64)) for g in grads) / 32, rel=1e-6)


def test_range_gaussian_gives_tp_sigma_and_clamp_rate_p():
    B = 1 << 16
    P = _params(d=B, block=B, n=1)
    rng = np.random.default_rng(8)
    x = (rng.standard_normal(B) * 1e-3).astype(F32)
    M = o.prepare_range(P, [x])
    assert M[0] == pytest.approx(TP32 * 1e-3, rel=0.02)
    R = o.rht_blocks(x, o.rademacher_signs(P.seed, 0, 0, B), B)
    frac = np.mean(np.abs(R) > M[0])
    assert abs(frac - 1 / 32) < 5 * math.sqrt((1 / 32) / B)


# ------------------------------------------------------------------ stochastic quantization
def _quantize_points(P, y_values, h16, M=1.0):
    """Feed chosen grid positions y through quantize_rotated by inverting y = (x + M) * scale."""
    rM = np.full(P.K, M, dtype=F32)
    scale, _, _ = o.block_scalars(P, rM)
    R = (np.asarray(y_values, dtype=np.float64) / np.float64(scale[0]) - M).astype(F32)
    return o.quantize_rotated(P, R, rM, np.asarray(h16, dtype=np.uint32)), R, rM


def test_sq_exhaustive_probability_over_all_halfwords():
    # every one of the 2^16 random integers, for a few positions inside a few table cells
    P = _params(d=65536, block=65536, n=1)
    rM = np.full(1, 1.0, dtype=F32)
    scale, _, _ = o.block_scalars(P, rM)
    h = np.arange(65536, dtype=np.uint32)
    for y_target in (0.75, 1.5, 2.999, 13.25, 14.5, 27.1, 29.99, 4.0000005):
        R = np.full(65536, F32(y_target / float(scale[0]) - 1.0), dtype=F32)
        y = F32(F32(R[0] + F32(1.0)) * scale[0])                 # the position the oracle will see
        z = o.quantize_rotated(P, R, rM, h).astype(np.int64)
        z0 = max(i for i in range(16) if T430[i] <= math.floor(float(y)))
        lo, wd = T430[z0], T430[z0 + 1] - T430[z0]
        assert set(np.unique(z)) <= {z0, z0 + 1}                  # only the two bracketing values
        p_up = np.mean(z == z0 + 1)
        assert abs(p_up - (float(y) - lo) / wd) <= 2.0 ** -16    # SQ probability of Sec. 4.1
        # expected decoded value equals y: unbiased (Sec. 4.1)
        assert abs(np.mean(np.array(T430)[z]) - float(y)) <= wd * 2.0 ** -16


def test_sq_on_table_values_is_deterministic_and_ends_are_fixed():
    P = _params(d=16 * 64, block=16 * 64, n=1)
    rng = np.random.default_rng(0)
    y = np.repeat(np.array(T430, dtype=np.float64), 64)
    z, R, rM = _quantize_points(P, y, rng.integers(0, 65536, size=y.size), M=1.0)
    # positions computed from R may be off a table value by an ulp; only exact hits are deterministic
    scale, _, _ = o.block_scalars(P, rM)
    yy = ((R + F32(1.0)).astype(F32) * scale[0]).astype(F32)
    exact = yy == y.astype(F32)
    assert exact.sum() > 0.5 * y.size
    assert np.array_equal(np.array(T430)[z[exact].astype(int)], y[exact].astype(int))
    # clamping: anything beyond +-M lands on the first / last index whatever the random draw
    big = np.array([-5.0, -1.0, 1.0, 7.0] * 256, dtype=F32)
    zz = o.quantize_rotated(P, big, rM, rng.integers(0, 65536, size=1024).astype(np.uint32))
    assert np.array_equal(zz, np.array([0, 0, 15, 15] * 256, dtype=np.uint8))


def test_sq_unbiased_with_the_real_stream():
    # E[T[z]] = y over many counters of the actual Philox stream
    B = 1 << 18
    P = _params(d=B, block=B, n=1)
    rM = np.full(1, 2.0, dtype=F32)
    scale, _, _ = o.block_scalars(P, rM)
    h = o.sq_halfwords(P.seed, 0, 0, 0, B)
    for y_target in (0.4, 6.3, 13.6, 14.2, 28.0):
        R = np.full(B, F32(y_target / float(scale[0]) - 2.0), dtype=F32)
        y = float(F32(F32(R[0] + F32(2.0)) * scale[0]))
        z = o.quantize_rotated(P, R, rM, h).astype(int)
        vals = np.array(T430)[z]
        wd = vals.max() - vals.min() if vals.max() > vals.min() else 1
        assert abs(vals.mean() - y) < 5 * 0.5 * wd / math.sqrt(B)


def test_identity_table_is_uniform_sq():
    # g = 2^b - 1 with the identity table: non-uniform THC degenerates to uniform SQ (Sec. 4.3),
    # i.e. z = floor(y) + [u < frac(y)]
    b, g = 3, 7
    P = o.Params(d=4096, block=4096, n=1, b=b, g=g, t_p=TP32, seed=5, table=list(range(8)))
    rng = np.random.default_rng(4)
    rM = np.full(1, 1.0, dtype=F32)
    R = rng.uniform(-1, 1, size=4096).astype(F32)
    h = rng.integers(0, 65536, size=4096).astype(np.uint32)
    z = o.quantize_rotated(P, R, rM, h).astype(int)
    scale, _, _ = o.block_scalars(P, rM)
    y = ((R + F32(1.0)).astype(F32) * scale[0]).astype(np.float64)
    u = (h + 0.5) / 65536.0
    expect = np.minimum(np.floor(y) + (u < (y - np.floor(y))), g).astype(int)
    assert np.mean(z != expect) < 1e-3            # binary32 vs binary64 can differ only on razor-edge draws
    assert np.all(np.abs(z - expect) <= 1)


def test_all_zero_block_maps_to_index_zero_and_decodes_to_zero():
    P = _params(d=2048, block=1024, n=2)
    rM = np.array([0.0, 1.0], dtype=F32)
    R = np.zeros(2048, dtype=F32)
    z = o.quantize_rotated(P, R, rM, np.arange(2048, dtype=np.uint32) * 31 % 65536)
    assert np.all(z[:1024] == 0)
    Y = np.zeros(2048, dtype=np.uint8)
    out = o.decompress(P, 0, Y, np.array([0.0, 0.0], dtype=F32))
    assert np.all(out == 0)


# ------------------------------------------------------------------ packing
def test_pack_golden_bytes(golden_dir):
    for line in open(os.path.join(golden_dir, "pack_b4_example.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        b, idx, byts = [s.strip() for s in line.split(":")]
        z = np.array([int(v) for v in idx.split()], dtype=np.uint8)
        expect = np.array([int(v, 16) for v in byts.split()], dtype=np.uint8)
        assert np.array_equal(o.pack_indices(z, int(b)), expect)
        assert np.array_equal(o.unpack_indices(expect, int(b)), z)


@pytest.mark.parametrize("b", [1, 2, 4, 8])
def test_pack_round_trip_every_value_at_every_position(b):
    per = 8 // b
    for pos in range(per):
        for v in range(2 ** b):
            z = np.zeros(per * 3, dtype=np.uint8)
            z[per + pos] = v
            pk = o.pack_indices(z, b)
            assert pk[0] == 0 and pk[2] == 0 and pk[1] == (v << (pos * b))
            assert np.array_equal(o.unpack_indices(pk, b), z)


@pytest.mark.parametrize("w", list(range(1, 17)))
def test_pack_fields_any_width(w):
    # field j sits at stream bit j*w, least-significant bit first: check against Python big integers
    rng = np.random.default_rng(w)
    v = rng.integers(0, 1 << w, size=64, dtype=np.uint32)
    v[0], v[1] = (1 << w) - 1, 0
    big = 0
    for j, x in enumerate(v.tolist()):
        big |= x << (j * w)
    expect = np.frombuffer(big.to_bytes(64 * w // 8, "little"), dtype=np.uint8)
    pk = o.pack_fields(v, w)
    assert np.array_equal(pk, expect)
    assert np.array_equal(o.unpack_fields(pk, w), v)
    if w == 8:
        assert np.array_equal(pk, v.astype(np.uint8))
    if w == 16:
        assert np.array_equal(pk, v.astype("<u2").view(np.uint8))


# ------------------------------------------------------------------ lookup / aggregate / homomorphism
def test_paper_worked_table_examples(golden_dir):
    text = open(os.path.join(golden_dir, "paper_sec4_3_tables.txt")).read()
    assert "T2" in text
    # T2 = [0,1,3,4], g = 4 on [-1, 1]: three senders
    P = o.Params(d=8, block=8, n=3, b=2, g=4, t_p=TP32, seed=0, table=[0, 1, 3, 4])
    rM = np.array([1.0], dtype=F32)
    deq = o.dequantize_indices(P, np.arange(4, dtype=np.uint8).repeat(2), rM)[::2]
    assert deq.tolist() == [-1.0, -0.5, 0.5, 1.0]
    case1 = [np.full(8, 1, dtype=np.uint8)] * 3                   # (1,1,1)
    case2 = [np.full(8, 0, dtype=np.uint8)] * 2 + [np.full(8, 2, dtype=np.uint8)]   # (0,0,2)
    Y1 = o.aggregate(P, [o.pack_indices(z, 2) for z in case1])
    Y2 = o.aggregate(P, [o.pack_indices(z, 2) for z in case2])
    assert np.all(Y1 == 3) and np.all(Y2 == 3)                    # same table-value sum ...
    for case in (case1, case2):                                   # ... same value sum -3/2
        tot = sum(o.dequantize_indices(P, z, rM).astype(np.float64) for z in case)
        assert np.all(tot == -1.5)
    assert sum(int(z[0]) for z in case1) != sum(int(z[0]) for z in case2)   # index sums differ
    # decompress-affine of the sum equals the average of decoded values: -1/2
    _, _, step_n = o.block_scalars(P, rM)
    assert F32(F32(3) * step_n[0]) + F32(-1.0) == F32(-0.5)
    # T0 (uniform): index sums determine value sums; T1 (non-uniform values, index sums) does not
    T0 = [Fraction(-1), Fraction(-1, 3), Fraction(1, 3), Fraction(1)]
    T1 = [Fraction(-1), Fraction(-1, 2), Fraction(1, 2), Fraction(1)]
    assert T0[0] + T0[3] == T0[1] + T0[2] == 0
    assert T1[1] + T1[3] == Fraction(1, 2) and T1[2] + T1[2] == 1
    # T0 expressed as an identity table with g = 3 decodes to those values
    P0 = o.Params(d=4, block=4, n=1, b=2, g=3, t_p=TP32, seed=0, table=[0, 1, 2, 3])
    d0 = o.dequantize_indices(P0, np.arange(4, dtype=np.uint8), rM).astype(np.float64)
    assert np.allclose(d0, [float(v) for v in T0], atol=1e-7)


def test_aggregate_is_the_naive_table_sum_and_max_case_fits():
    P = _params(d=4096, block=1024, n=8)
    rng = np.random.default_rng(6)
    zs = [rng.integers(0, 16, size=4096).astype(np.uint8) for _ in range(8)]
    Y = o.aggregate(P, [o.pack_indices(z, 4) for z in zs])
    naive = [sum(T430[int(z[j])] for z in zs) for j in range(0, 4096, 37)]
    assert Y[::37].tolist() == naive
    top = [np.full(4096, 15, dtype=np.uint8)] * 8
    Ymax = o.aggregate(P, [o.pack_indices(z, 4) for z in top])
    assert Ymax.dtype == np.uint8 and np.all(Ymax == 240)          # g*n = 240 < 256 (Sec. 8 setup)
    with pytest.raises(AssertionError):
        _params(n=9)                                               # 270 does not fit 8 bits
    P16 = _params(d=4096, block=1024, n=16, agg_bits=16)
    Y16 = o.aggregate(P16, [o.pack_indices(np.full(4096, 15, dtype=np.uint8), 4)] * 16)
    assert Y16.dtype == np.uint16 and np.all(Y16 == 480)


def test_table_precondition_is_enforced():
    with pytest.raises(AssertionError):
        o.Params(d=8, block=8, n=1, b=2, g=4, t_p=TP32, seed=0, table=[0, 3, 1, 4])
    with pytest.raises(AssertionError):
        o.Params(d=8, block=8, n=1, b=2, g=4, t_p=TP32, seed=0, table=[1, 2, 3, 4])


def test_homomorphism_identity():
    # D( (1/n) sum_i T(C(x_i)) ) = (1/n) sum_i D(T(C(x_i)))   (Sec. 4.3)
    P = _params(d=8192, block=1024, n=5, agg_bits=8)
    rng = np.random.default_rng(12)
    grads = [(rng.standard_normal(8192) * 10 ** rng.uniform(-4, -2)).astype(F32) for _ in range(5)]
    M, packed, Y, out, _ = o.thc_round(P, 3, grads)
    zs = [o.unpack_indices(pk, 4) for pk in packed]
    assert np.array_equal(Y.astype(np.int64), sum(np.array(T430)[z.astype(int)] for z in zs))
    mean_deq = sum(o.dequantize_indices(P, z, M).astype(np.float64) for z in zs) / 5
    _, _, step_n = o.block_scalars(P, M)
    v = (Y.astype(F32) * np.repeat(step_n, 1024)).astype(F32) + (-np.repeat(M, 1024))
    assert np.max(np.abs(v.astype(np.float64) - mean_deq)) <= 4e-7 * float(M.max())
    # and after the (linear) inverse rotation
    signs = o.rademacher_signs(P.seed, 3, 0, 8192)
    mean_out = sum(o.irht_blocks(o.dequantize_indices(P, z, M), signs, 1024).astype(np.float64) for z in zs) / 5
    assert np.linalg.norm(out - mean_out) <= 1e-6 * np.linalg.norm(mean_out)


# ------------------------------------------------------------------ end to end
def test_round_trip_nmse_matches_theory():
    # One worker, Gaussian input: NMSE = cost(T) (quantization) + truncation term, in sigma^2 units
    B = 1 << 16
    P = _params(d=4 * B, block=B, n=1)
    rng = np.random.default_rng(21)
    x = (rng.standard_normal(4 * B) * 3e-3).astype(F32)
    _, _, _, out, _ = o.thc_round(P, 0, [x])
    tp = TP32
    trunc = 2 * ((1 + tp * tp) * scipy.stats.norm.sf(tp) - tp * scipy.stats.norm.pdf(tp))
    expect = o.table_cost(T430, 30, tp) + trunc
    assert o.nmse(x, out) == pytest.approx(expect, rel=0.05)
    # identical copies on n workers: independent rounding noise averages out ~ 1/n, truncation bias stays
    n = 8
    Pn = _params(d=4 * B, block=B, n=n)
    _, _, _, outn, _ = o.thc_round(Pn, 0, [x] * n)
    assert o.nmse(x, outn) == pytest.approx(o.table_cost(T430, 30, tp) / n + trunc, rel=0.08)


def test_error_feedback_identity_and_carry_over():
    P = _params(d=4096, block=1024, n=2)
    rng = np.random.default_rng(31)
    grads = [rng.standard_normal(4096).astype(F32) * F32(1e-2) for _ in range(2)]
    efs = [np.zeros(4096, dtype=F32) for _ in range(2)]
    M, packed, Y, out, new_efs = o.thc_round(P, 0, grads, efs)
    signs = o.rademacher_signs(P.seed, 0, 0, 4096)
    for i in range(2):
        X = o.dequantize_indices(P, o.unpack_indices(packed[i], 4), M)
        rec = o.irht_blocks(X, signs, 1024)
        # x = e' + RHT^-1(X)   (Alg. 3, error-feedback update)
        assert np.allclose(new_efs[i].astype(np.float64) + rec, grads[i], atol=1e-7)
        assert 0 < np.linalg.norm(new_efs[i]) < 0.5 * np.linalg.norm(grads[i])
    # next round sends grad + e
    M2, packed2, _, _, _ = o.thc_round(P, 1, grads, new_efs)
    Mplain = o.prepare_range(P, grads)
    assert not np.array_equal(M2, Mplain)


def test_bf16_inputs_are_widened_exactly():
    import torch
    t = torch.randn(1024, dtype=torch.float32).to(torch.bfloat16)
    as_f32 = t.to(torch.float32).numpy()
    bits = t.view(torch.int16).numpy().astype(np.uint16).astype(np.uint32) << 16
    assert np.array_equal(bits.view(np.float32), as_f32)
    assert np.array_equal(o.ef_input(as_f32, None), as_f32)


# ------------------------------------------------------------------ table solver (Sec. 5.2, App. B)
def test_tp_definition():
    assert TP32 == pytest.approx(scipy.stats.norm.ppf(1 - 1 / 64), rel=1e-12)
    assert 2 * scipy.stats.norm.sf(TP32) == pytest.approx(1 / 32, rel=1e-9)


def test_pair_cost_closed_form_matches_quadrature_of_literal_objective():
    # the literal integrand: P(a,q0)(a-q0)^2 + P(a,q1)(a-q1)^2 with SQ probabilities (Sec. 5.2)
    for q0, q1 in [(-2.1, -1.3), (-0.4, 0.9), (0.0, 0.1), (1.0, 2.15)]:
        def f(a):
            p1 = (a - q0) / (q1 - q0)
            return (p1 * (a - q1) ** 2 + (1 - p1) * (a - q0) ** 2) * scipy.stats.norm.pdf(a)
        ref, _ = scipy.integrate.quad(f, q0, q1, epsabs=1e-14, epsrel=1e-12)
        assert o.pair_cost(q0, q1) == pytest.approx(ref, rel=1e-9, abs=1e-14)


def test_worked_integral_of_appendix_b():
    # b = 2, g = 4, T = [0, 1, 3, 4]: the three integrals written out in App. B
    tp = TP32
    pdf = scipy.stats.norm.pdf
    i1, _ = scipy.integrate.quad(lambda a: ((a + tp) / (tp / 2) * (a + tp / 2) ** 2
                                            + (-tp / 2 - a) / (tp / 2) * (a + tp) ** 2) * pdf(a), -tp, -tp / 2)
    i2, _ = scipy.integrate.quad(lambda a: ((a + tp / 2) / tp * (a - tp / 2) ** 2
                                            + (tp / 2 - a) / tp * (a + tp / 2) ** 2) * pdf(a), -tp / 2, tp / 2)
    i3, _ = scipy.integrate.quad(lambda a: ((a - tp / 2) / (tp / 2) * (a - tp) ** 2
                                            + (tp - a) / (tp / 2) * (a - tp / 2) ** 2) * pdf(a), tp / 2, tp)
    assert o.table_cost([0, 1, 3, 4], 4, tp) == pytest.approx(i1 + i2 + i3, rel=1e-9)


def test_stars_and_bars_enumeration_counts_and_distinct():
    for n, k in [(0, 3), (3, 1), (4, 3), (5, 4), (7, 7)]:
        items = [tuple(B) for B in o.stars_and_bars(n, k)]
        assert len(items) == math.comb(n + k - 1, k - 1)
        assert len(set(items)) == len(items)
        assert all(sum(B) == n and min(B) >= 0 for B in items)
    # the count quoted in App. B for b = 4, g = 51 under the symmetry constraint
    assert math.comb(23, 6) == 100947
    # number of strictly increasing tables from 0 to g
    for b, g in [(2, 4), (2, 8), (3, 10)]:
        assert sum(1 for _ in o.enumerate_tables(b, g)) == math.comb(g - 1, 2 ** b - 2)


@pytest.mark.parametrize("b,g", [(1, 1), (1, 5), (2, 3), (2, 4), (2, 5), (2, 8), (2, 9), (2, 12), (3, 7), (3, 9),
                                  (3, 10), (3, 12), (3, 13)])
def test_solver_equals_brute_force(b, g):
    p = 1 / 32
    tp = o.t_p_of(p)
    best, best_cost = None, math.inf
    for T in o.enumerate_tables(b, g):
        c = o.table_cost(T, g, tp)
        if best is None or c < best_cost - 1e-12 * abs(best_cost) \
                or (abs(c - best_cost) <= 1e-12 * abs(best_cost) and T < best):
            best, best_cost = T, c
    got = o.solve_table(b, g, p)
    assert o.table_cost(got, g, tp) == pytest.approx(best_cost, rel=1e-12)
    assert got == best


def test_solver_special_cases():
    assert o.solve_table(4, 15, 1 / 32) == list(range(16))         # g = 2^b - 1: identity (Sec. 4.3)
    assert o.solve_table(2, 3, 1 / 1024) == [0, 1, 2, 3]
    for b, g, p in [(4, 51, 1 / 32), (4, 31, 1 / 32), (2, 9, 1 / 32)]:
        T = o.solve_table(b, g, p)                                   # odd g: mirror-symmetric optimum (App. B)
        assert [g - v for v in reversed(T)] == T
    # The objective is mirror-symmetric, so the mirror of an optimum is an optimum; App. B goes further and
    # assumes the optimum itself is symmetric for odd g.  That fails for some (b, g, p): the exact optimum is then
    # an asymmetric table tied with its mirror, and strictly better than the best symmetric table.
    for b, g, p in [(3, 21, 1 / 1024), (4, 51, 1 / 1024)]:
        T = o.solve_table(b, g, p)
        mirror = [g - v for v in reversed(T)]
        tp = o.t_p_of(p)
        assert mirror != T and T < mirror
        assert o.table_cost(mirror, g, tp) == pytest.approx(o.table_cost(T, g, tp), rel=1e-12)
    sym_best = min((T for T in o.enumerate_tables(3, 21) if [21 - v for v in reversed(T)] == T),
                   key=lambda T: o.table_cost(T, 21, o.t_p_of(1 / 1024)))
    assert o.table_cost(sym_best, 21, o.t_p_of(1 / 1024)) > \
        o.table_cost(o.solve_table(3, 21, 1 / 1024), 21, o.t_p_of(1 / 1024)) * (1 + 1e-9)
    T = o.solve_table(4, 30, 1 / 32)
    assert T == T430
    mirror = [30 - v for v in reversed(T)]
    assert mirror != T and mirror > T                                # tie broken towards the smaller table
    assert o.table_cost(mirror, 30, TP32) == pytest.approx(o.table_cost(T, 30, TP32), rel=1e-12)
    assert o.solve_table(2, 8, 1 / 32) == [0, 3, 5, 8]
    # finer grids never hurt when they refine the coarse grid
    assert o.table_cost(o.solve_table(4, 30, 1 / 32), 30, TP32) <= o.table_cost(list(range(16)), 15, TP32)


def test_a_slice_with_its_offset_reproduces_the_whole_vector():
    """Blocks are independent instances and the random streams are indexed by global coordinate: compressing and
    decompressing blocks [2, 5) on their own, with j0 = 2 B, gives the bytes of the whole-vector result."""
    B, K, n = 1024, 5, 3
    P = _params(d=B * K, block=B, n=n)
    rng = np.random.default_rng(11)
    grads = [rng.standard_normal(P.d).astype(np.float32) * 1e-3 for _ in range(n)]
    efs = [rng.standard_normal(P.d).astype(np.float32) * 1e-4 for _ in range(n)]
    M, packed, Y, out, new_efs = o.thc_round(P, 4, grads, efs)
    lo, hi = 2 * B, 5 * B
    Ps = _params(d=hi - lo, block=B, n=n)
    Ms = o.prepare_range(Ps, [g[lo:hi] for g in grads], [e[lo:hi] for e in efs])
    assert np.array_equal(Ms, M[2:5])
    pks = []
    for i in range(n):
        pk, ne = o.compress(Ps, i, 4, grads[i][lo:hi], efs[i][lo:hi], Ms, j0=lo)
        assert np.array_equal(pk, packed[i][lo // 2:hi // 2]) and np.array_equal(ne, new_efs[i][lo:hi])
        pks.append(pk)
    Ys = o.aggregate(Ps, pks)
    assert np.array_equal(Ys, Y[lo:hi])
    assert np.array_equal(o.decompress(Ps, 4, Ys, Ms, j0=lo), out[lo:hi])
    # and the offset matters: the same slice taken for the start of a vector uses other random draws
    pk0, _ = o.compress(Ps, 0, 4, grads[0][lo:hi], efs[0][lo:hi], Ms, j0=0)
    assert not np.array_equal(pk0, pks[0])


def test_power_of_two_scaling_leaves_the_indices_alone_down_to_where_the_scale_overflows():
    """Every step up to the index is homogeneous of degree one or zero in the input, and scaling by a power of two
    is exact in binary32: the packed bytes must not change and the estimate must scale exactly.  That holds down to
    the point where g / (M - m) no longer is a finite binary32 number: from there on the block counts as empty."""
    P = _params(d=2048, block=1024, n=2)
    rng = np.random.default_rng(5)
    grads = [rng.standard_normal(P.d).astype(np.float32) * 1e-3 for _ in range(P.n)]
    M, packed, Y, out, _ = o.thc_round(P, 1, grads)
    for k in (-40, 30, -80, -100, -110, -115):
        s = np.float32(2.0 ** k)
        Ms, packed_s, Ys, out_s, _ = o.thc_round(P, 1, [g * s for g in grads])
        assert np.array_equal(Ms, M * s)
        assert np.all(np.isfinite(np.float64(P.g) / (2.0 * Ms.astype(np.float64))).astype(bool))
        assert all(np.array_equal(a, b) for a, b in zip(packed_s, packed)), k
        assert np.array_equal(Ys, Y)
        if k >= -100:                      # below that the smallest outputs are subnormal and round
            assert np.array_equal(out_s, out * s)
    # M = 2.7e-38: g / (2 M) = 5.6e38 is beyond binary32: the block is empty, all indices are 0 and it decodes to
    # m = -M in the rotated domain
    s = np.float32(2.0 ** -116)
    Ms, packed_s, Ys, _, _ = o.thc_round(P, 1, [g * s for g in grads])
    with np.errstate(over="ignore"):
        assert np.all(Ms > 0) and np.all(np.isinf((np.float64(P.g) / (2.0 * Ms.astype(np.float64))).astype(np.float32)))
    assert all(not pk.any() for pk in packed_s) and not Ys.any()
