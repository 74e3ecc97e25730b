"""Pins for the oracle's uniform THC (Alg. 1, Sec. 4.2, App. A): identities and examples the paper states."""
import numpy as np
import pytest

from oracle import thc_oracle as o

F32 = np.float32
TP32 = o.t_p_of(1 / 32)


def uparams(d, block, n, b, agg_bits=8, seed=11):
    return o.Params(d=d, block=block, n=n, b=b, g=2 ** b - 1, t_p=TP32, seed=seed, table=list(range(2 ** b)),
                    agg_bits=agg_bits)


def test_general_range_reduces_to_the_symmetric_one():
    P = o.Params(d=4096, block=1024, n=1, b=4, g=30, t_p=TP32, seed=3,
                 table=[0, 3, 5, 7, 9, 11, 13, 14, 15, 17, 19, 21, 23, 25, 27, 30])
    rng = np.random.default_rng(0)
    R = rng.standard_normal(4096).astype(F32)
    M = rng.uniform(1, 3, size=4).astype(F32)
    h = rng.integers(0, 65536, size=4096).astype(np.uint32)
    z0 = o.quantize_rotated(P, R, M, h)
    z1 = o.quantize_rotated(P, R, M, h, range_m=-M)
    assert np.array_equal(z0, z1)
    assert np.array_equal(o.dequantize_indices(P, z0, M), o.dequantize_indices(P, z0, M, -M))
    for a, b_ in zip(o.block_scalars(P, M), o.block_scalars(P, M, -M)):
        assert np.array_equal(a, b_)


def test_uniform_levels_of_the_papers_four_value_example():
    # Sec. 4.3: USQ of [-1, 1] with four values uses -1, -1/3, 1/3, 1
    P = uparams(8, 8, 1, 2)
    m, M = np.array([-1.0], dtype=F32), np.array([1.0], dtype=F32)
    deq = o.dequantize_indices(P, np.array([0, 1, 2, 3, 0, 1, 2, 3], dtype=np.uint8), M, m)
    assert np.allclose(deq[:4], [-1, -1 / 3, 1 / 3, 1], atol=1e-7)
    # the value 0 lies midway between -1/3 and 1/3: it goes up for (almost exactly) half of all draws
    Pbig = uparams(65536, 65536, 1, 2)
    z = o.quantize_rotated(Pbig, np.zeros(65536, dtype=F32), M, np.arange(65536, dtype=np.uint32), m)
    assert set(np.unique(z)) == {1, 2} and abs(np.mean(z == 2) - 0.5) <= 2.0 ** -15


def test_extremes_and_unbiasedness():
    b, n, d = 3, 1, 1 << 16
    P = uparams(d, d, n, b)
    rng = np.random.default_rng(5)
    x = rng.uniform(-0.3, 0.9, size=d).astype(F32)
    m, M = o.uniform_range(P, 0, [x], None, rotate=False)
    assert m[0] == x.min() and M[0] == x.max()
    pk, _ = o.uniform_compress(P, 0, 0, x, None, m, M, rotate=False)
    z = o.unpack_indices(pk, b)
    assert z[np.argmin(x)] == 0                                   # the minimum is a quantization value
    assert z[np.argmax(x)] in (2 ** b - 2, 2 ** b - 1)            # the maximum, up to one rounding of the scale
    deq = o.dequantize_indices(P, z, M, m).astype(np.float64)
    step = (float(M[0]) - float(m[0])) / (2 ** b - 1)
    assert np.all(np.abs(deq - x) <= step * (1 + 1e-6))          # only the two neighbouring values
    assert abs(np.mean(deq - x)) < 5 * step / np.sqrt(12 * d) * 2  # unbiased (Sec. 4.1)


def test_homomorphic_usq_identity():
    # Sec. 4.2: (1/n) sum_i D(C(x_i)) = D((1/n) sum_i C(x_i)) when all workers share [m, M]
    b, n, d, block = 4, 6, 4096, 1024
    P = uparams(d, block, n, b)
    rng = np.random.default_rng(2)
    grads = [(rng.standard_normal(d) * (1 + i)).astype(F32) for i in range(n)]
    m, M = o.uniform_range(P, 4, grads, None, rotate=False)
    for k in range(d // block):
        allv = np.stack([g[k * block:(k + 1) * block] for g in grads])
        assert m[k] == allv.min() and M[k] == allv.max()          # global extremes, not per worker
    packed = [o.uniform_compress(P, i, 4, grads[i], None, m, M, rotate=False)[0] for i in range(n)]
    Y = o.aggregate(P, packed)                                    # identity table: the sum of the indices
    assert np.array_equal(Y.astype(np.int64), sum(o.unpack_indices(pk, b).astype(np.int64) for pk in packed))
    est = o.uniform_decompress(P, 4, Y, m, M, rotate=False).astype(np.float64)
    mean_deq = sum(o.dequantize_indices(P, o.unpack_indices(pk, b), M, m).astype(np.float64) for pk in packed) / n
    assert np.max(np.abs(est - mean_deq)) <= 1e-6 * float(np.max(M - m))
    # Alg. 1's last line, literally: m + (1/n) X (M - m) / (2^b - 1)
    k = 0
    lit = float(m[k]) + Y[:block].astype(np.float64) / n * (float(M[k]) - float(m[k])) / (2 ** b - 1)
    assert np.max(np.abs(est[:block] - lit)) <= 1e-6 * float(M[k] - m[k])


def test_appendix_a_bad_case_and_what_rotation_buys():
    # App. A: b = 1 and the vector (1, -1, 0, ..., 0): every zero is rounded with an error of 1
    d = 1 << 12
    P = uparams(d, d, 1, 1)
    x = np.zeros(d, dtype=F32)
    x[0], x[1] = 1.0, -1.0
    m, M = o.uniform_range(P, 0, [x], None, rotate=False)
    assert (m[0], M[0]) == (-1.0, 1.0)
    pk, _ = o.uniform_compress(P, 0, 0, x, None, m, M, rotate=False)
    est = o.uniform_decompress(P, 0, o.aggregate(P, [pk]), m, M, rotate=False)
    assert np.all(np.abs(est[2:]) == 1.0) and est[0] == 1.0 and est[1] == -1.0
    nmse_plain = o.nmse(x, est)
    assert nmse_plain == pytest.approx((d - 2) / 2)
    # with the rotation the range shrinks from 2 to O(sqrt(log d / d)) (Sec. 5.1) and so does the error
    m2, M2 = o.uniform_range(P, 0, [x], None, rotate=True)
    assert (M2[0] - m2[0]) < 0.1
    pk2, _ = o.uniform_compress(P, 0, 0, x, None, m2, M2, rotate=True)
    est2 = o.uniform_decompress(P, 0, o.aggregate(P, [pk2]), m2, M2, rotate=True)
    assert o.nmse(x, est2) < nmse_plain / 500


def test_uniform_error_feedback_identity():
    b, n, d, block = 2, 2, 2048, 1024
    P = uparams(d, block, n, b)
    rng = np.random.default_rng(9)
    grads = [rng.standard_normal(d).astype(F32) for _ in range(n)]
    efs = [(rng.standard_normal(d) * 0.1).astype(F32) for _ in range(n)]
    for rotate in (False, True):
        m, M = o.uniform_range(P, 1, grads, efs, rotate)
        for i in range(n):
            pk, ne = o.uniform_compress(P, i, 1, grads[i], efs[i], m, M, rotate)
            X = o.dequantize_indices(P, o.unpack_indices(pk, b), M, m)
            if rotate:
                X = o.irht_blocks(X, o.rademacher_signs(P.seed, 1, 0, d), block)
            assert np.allclose(ne.astype(np.float64) + X, (grads[i] + efs[i]).astype(np.float64), atol=1e-6)
