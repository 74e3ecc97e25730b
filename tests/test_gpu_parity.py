"""Parity of the HIP library (through the C-ABI binding) against the CPU oracle, element by element,
on the same seeded inputs.  Bars:
  * packed bytes, aggregated sums: bit-exact, except that at most 1e-6 of the indices may differ, by one
    level, where a value sits within an ulp of a rounding threshold (expected: none);
  * float outputs (decompressed average, error-feedback buffers): relative L2 error <= 1e-5
    (expected: bit-identical, the butterfly order is fixed);
  * range M: relative error <= 2^-23 (binary64 sums in a different order, rounded once to binary32).
"""
import numpy as np
import pytest
import torch

from oracle import thc_oracle as o
from paper_2302_08545_amd import api
from paper_2302_08545_amd import workloads as wl

pytestmark = pytest.mark.gpu

DEV = "cuda:0"
SEED = wl.RHT_SEED
F32 = np.float32


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the GPU"
    api.lib()
    yield
    torch.cuda.synchronize()


def table_for(b, g, p=1 / 32):
    return o.solve_table(b, g, p)


def both_params(d, block, n, b=4, g=30, agg_bits=8, p=1 / 32, bf16=False, seed=SEED, table=None, order=0,
                first_block=0, group_log2=0, single_launch=0):
    T = table if table is not None else table_for(b, g, p)
    tp = o.t_p_of(p)
    P = o.Params(d=d, block=block, n=n, b=b, g=g, t_p=tp, seed=seed, table=T, agg_bits=agg_bits, order=order)
    L = api.make_params(d, block, n, b, g, tp, seed, T, agg_bits, api.THC_DTYPE_BF16 if bf16 else api.THC_DTYPE_F32,
                        order, first_block, group_log2, single_launch)
    return P, L


def rel_l2(a, b):
    a = a.astype(np.float64)
    b = b.astype(np.float64)
    nb = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / nb) if nb > 0 else float(np.linalg.norm(a))


def assert_indices_match(gpu_packed, ref_packed, b, label=""):
    if np.array_equal(gpu_packed, ref_packed):
        return
    zg = o.unpack_indices(gpu_packed, b).astype(np.int64)
    zr = o.unpack_indices(ref_packed, b).astype(np.int64)
    diff = zg != zr
    assert diff.mean() <= 1e-6 and np.abs(zg - zr).max() <= 1, \
        f"{label}: {diff.sum()} of {diff.size} indices differ, max step {np.abs(zg - zr).max()}"


class GpuRound:
    """Device buffers for one configuration and the calls on them."""

    def __init__(self, L, ef=False):
        self.L = L
        d, n = L.d, L.n
        self.K = d // L.block
        self.ws = torch.zeros(api.thc_workspace_bytes(L, ef), dtype=torch.uint8, device=DEV)
        self.range_M = torch.zeros(self.K, dtype=torch.float32, device=DEV)
        self.packed = [torch.zeros(d * L.b // 8, dtype=torch.uint8, device=DEV) for _ in range(n)]
        self.agg = torch.zeros(d * L.agg_bits // 8, dtype=torch.uint8, device=DEV)
        self.out = torch.zeros(d, dtype=torch.float32, device=DEV)
        self.efs = [torch.zeros(d, dtype=torch.float32, device=DEV) for _ in range(n)] if ef else None

    def prepare(self, grads):
        """thc_prepare_range: the norms and the range, nothing else."""
        api.thc_prepare_range(self.L, grads, self.efs, self.range_M, self.ws)

    def compress_each(self, rnd, grads, range_M=None):
        """n calls of thc_compress (one worker each), with this object's range or the caller's."""
        rm = self.range_M if range_M is None else range_M
        for i in range(self.L.n):
            api.thc_compress(self.L, i, rnd, grads[i], None if self.efs is None else self.efs[i], rm,
                             self.packed[i], self.ws)

    def compress_all(self, rnd, grads):
        """thc_compress_all: range and all n workers' streams in one sweep."""
        api.thc_compress_all(self.L, rnd, grads, self.efs, self.range_M, self.packed, self.ws)

    def status(self):
        """Status word of the last single-launch sweep on this workspace (0 = fine)."""
        torch.cuda.synchronize()
        return int(self.ws[:4].view(torch.int32).cpu()[0])

    def aggregate(self):
        api.thc_aggregate(self.L, self.packed, self.agg)

    def decompress(self, rnd, range_M=None):
        api.thc_decompress(self.L, rnd, self.agg, self.range_M if range_M is None else range_M, self.out, self.ws)

    def agg_numpy(self):
        a = self.agg.cpu().numpy()
        if self.L.agg_bits == 8:
            return a
        if self.L.agg_bits == 16:
            return a.view(np.uint16)
        return o.unpack_fields(a, self.L.agg_bits)


def make_grads(d, n, scale=1e-3, seed=1, bf16=False):
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    out = []
    for i in range(n):
        t = torch.randn(d, generator=g, dtype=torch.float32) * (scale * (1 + 0.3 * i))
        if bf16:
            t = t.to(torch.bfloat16)
        out.append(t)
    return out


def to_np32(t):
    return t.to(torch.float32).cpu().numpy()


# ----------------------------------------------------------------------------- individual calls
@pytest.mark.parametrize("block,K,n", [(1 << 10, 3, 2), (1 << 11, 5, 2), (1 << 12, 4, 3), (1 << 13, 3, 2),
                                       (1 << 15, 2, 2), (1 << 20, 2, 4),
                                       # whole spans of 2^19 coordinates: the first pass permutes its tile order
                                       (1 << 12, 128, 2), (1 << 10, 1024, 1), (1 << 15, 48, 1), (1 << 13, 192, 1)])
def test_prepare_range_and_compress(block, K, n):
    d = block * K
    P, L = both_params(d, block, n)
    grads = make_grads(d, n, seed=block + K)
    grads[0][:block] *= 30.0                     # a block where one worker dominates the norm
    R = GpuRound(L)
    dg = [g.to(DEV) for g in grads]
    R.prepare(dg)
    M_ref = o.prepare_range(P, [to_np32(g) for g in grads])
    M_gpu = R.range_M.cpu().numpy()
    assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23), (M_gpu, M_ref)
    # the oracle's range goes into the GPU's compress, so a last-bit difference in M cannot hide anything
    R.compress_each(4, dg, range_M=torch.from_numpy(M_ref).to(DEV))
    for i in range(n):
        ref, _ = o.compress(P, i, 4, to_np32(grads[i]), None, M_ref)
        assert_indices_match(R.packed[i].cpu().numpy(), ref, L.b, f"worker {i}")


@pytest.mark.parametrize("b,g,agg_bits,n", [(4, 30, 8, 8), (4, 30, 8, 1), (4, 30, 8, 3), (4, 30, 16, 16), (2, 8, 8, 16),
                                            (4, 15, 8, 17), (1, 1, 8, 64), (8, 255, 16, 5), (2, 3, 16, 64), (4, 36, 16, 64),
                                            (3, 12, 8, 10), (3, 7, 6, 9), (4, 30, 7, 4), (4, 30, 9, 16), (5, 40, 11, 33),
                                            (2, 8, 7, 15), (6, 63, 13, 64), (7, 200, 16, 9), (1, 1, 1, 1), (4, 30, 5, 1),
                                            (4, 255, 16, 7), (4, 100, 16, 64), (4, 128, 16, 3), (4, 85, 16, 10),
                                            (2, 8, 8, 1), (2, 3, 8, 64), (2, 8, 8, 31), (2, 255, 8, 1)])
def test_aggregate_bit_exact(b, g, agg_bits, n):
    d = 5 * 1024
    T = table_for(b, g) if g > 2 ** b - 1 else list(range(2 ** b))
    P, L = both_params(d, 1024, n, b=b, g=g, agg_bits=agg_bits, table=T)
    rng = np.random.default_rng(b * 100 + n)
    packed = [rng.integers(0, 256, size=d * b // 8, dtype=np.uint8) for _ in range(n)]
    if n >= 2:
        packed[0][:] = 0xFF                      # every index at the top: exercises the largest sums
        packed[1][: d * b // 16] = 0xFF
    R = GpuRound(L)
    for i in range(n):
        R.packed[i].copy_(torch.from_numpy(packed[i]))
    R.aggregate()
    ref = o.aggregate(P, packed)
    assert np.array_equal(R.agg_numpy(), ref)
    assert np.array_equal(R.agg.cpu().numpy(), o.aggregate_stream(P, ref))     # the bytes a PS would send


def test_aggregate_all_top_indices_reach_g_times_n():
    P, L = both_params(4096, 1024, 8)
    R = GpuRound(L)
    for t in R.packed:
        t.fill_(0xFF)
    R.aggregate()
    assert np.all(R.agg_numpy() == 240)          # g*n = 240 fits 8 bits (Sec. 8 setup)


@pytest.mark.parametrize("block,K,agg_bits,n", [(1 << 10, 3, 8, 4), (1 << 12, 2, 16, 12), (1 << 13, 2, 8, 8), (1 << 16, 2, 8, 2),
                                                (1 << 20, 1, 8, 8), (1 << 11, 3, 7, 4), (1 << 13, 2, 9, 16), (1 << 14, 1, 12, 40),
                                                (1 << 11, 512, 8, 3), (1 << 14, 96, 8, 2)])
def test_decompress(block, K, agg_bits, n):
    d = block * K
    P, L = both_params(d, block, n, agg_bits=agg_bits)
    rng = np.random.default_rng(d + n)
    Y = rng.integers(0, 30 * n + 1, size=d).astype(np.uint8 if agg_bits <= 8 else np.uint16)
    M = (rng.uniform(0.5, 2.0, size=K) * 1e-3).astype(F32)
    R = GpuRound(L)
    R.agg.copy_(torch.from_numpy(o.aggregate_stream(P, Y)))
    R.decompress(9, range_M=torch.from_numpy(M).to(DEV))
    ref = o.decompress(P, 9, Y, M)
    got = R.out.cpu().numpy()
    assert rel_l2(got, ref) <= 1e-5
    assert np.array_equal(got, ref), "fixed butterfly order should make this bit-identical"


# ----------------------------------------------------------------------------- whole rounds
@pytest.mark.parametrize("block,K,n,b,g,agg_bits", [(1 << 10, 9, 4, 4, 30, 8), (1 << 14, 2, 8, 4, 30, 8), (1 << 20, 1, 4, 4, 30, 8),
                                                    (1 << 12, 3, 16, 2, 8, 8), (1 << 12, 3, 16, 4, 30, 16), (1 << 11, 4, 2, 1, 1, 8),
                                                    (1 << 13, 2, 3, 8, 255, 16), (1 << 14, 2, 10, 3, 12, 7), (1 << 10, 5, 16, 4, 30, 9),
                                                    (1 << 15, 1, 5, 6, 100, 10), (1 << 12, 2, 4, 3, 7, 5)])
def test_full_round_on_gpu_ranges(block, K, n, b, g, agg_bits):
    """thc_prepare_range, thc_compress_all, thc_aggregate, thc_decompress with the GPU's own range: the two range
    calls agree bit for bit, the range is within 2^-23 of the oracle's, and everything after it equals the oracle
    working from that very range."""
    d = block * K
    T = table_for(b, g) if g > 2 ** b - 1 else list(range(2 ** b))
    P, L = both_params(d, block, n, b=b, g=g, agg_bits=agg_bits, table=T)
    grads = make_grads(d, n, seed=7 * n + b)
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    R.prepare(dg)
    M_prep = R.range_M.clone()
    R.compress_all(2, dg)
    assert torch.equal(R.range_M, M_prep)
    R.aggregate()
    R.decompress(2)
    M_ref = o.prepare_range(P, gn)
    M_gpu = R.range_M.cpu().numpy()
    assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    packed = [o.compress(P, i, 2, gn[i], None, M_gpu)[0] for i in range(n)]
    for i in range(n):
        assert_indices_match(R.packed[i].cpu().numpy(), packed[i], b, f"worker {i}")
    Y = o.aggregate(P, packed)
    assert np.mean(R.agg_numpy() != Y) <= 1e-6 * n
    out = o.decompress(P, 2, Y, M_gpu)
    assert rel_l2(R.out.cpu().numpy(), out) <= 1e-5
    mean = np.mean([x.astype(np.float64) for x in gn], axis=0)
    assert o.nmse(mean, R.out.cpu().numpy()) == pytest.approx(o.nmse(mean, out), rel=0.02)


def test_error_feedback_rounds():
    """Two rounds with error feedback: e' = (grad + e) - RHT^-1(X_i), carried into the next round."""
    block, K, n = 1 << 12, 3, 3
    d = block * K
    P, L = both_params(d, block, n)
    R = GpuRound(L, ef=True)
    efs_ref = [np.zeros(d, dtype=F32) for _ in range(n)]
    for rnd in range(2):
        grads = make_grads(d, n, seed=40 + rnd)
        dg = [x.to(DEV) for x in grads]
        gn = [to_np32(x) for x in grads]
        M_ref = o.prepare_range(P, gn, efs_ref)
        R.prepare(dg)
        M_gpu = R.range_M.cpu().numpy()
        assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
        R.compress_each(rnd, dg, range_M=torch.from_numpy(M_ref).to(DEV))
        new_ref = []
        for i in range(n):
            pk, ne = o.compress(P, i, rnd, gn[i], efs_ref[i], M_ref)
            assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"round {rnd} worker {i}")
            got = R.efs[i].cpu().numpy()
            assert rel_l2(got, ne) <= 1e-5, f"round {rnd} worker {i}"
            new_ref.append(ne)
        efs_ref = new_ref
        for i in range(n):                       # keep both sides on exactly the same state
            R.efs[i].copy_(torch.from_numpy(efs_ref[i]))


@pytest.mark.parametrize("L,K,n,bf16,order", [(12, 11, 2, False, 0), (16, 5, 2, True, 1), (18, 3, 1, False, 1),
                                                 (21, 2, 1, False, 1)])
def test_piecewise_processing_matches_the_oracle(L, K, n, bf16, order):
    """Every call walks long vectors in groups of whole blocks that share the workspace's slot.  With the group forced
    down to 2^14 coordinates (or one block, if larger) these vectors take several groups, the last one shorter; packed
    bytes, error feedback and the output must not change."""
    block = 1 << L
    d = block * K
    P, Lp = both_params(d, block, n, bf16=bf16, order=order, group_log2=14)
    R = GpuRound(Lp, ef=True)
    efs_ref = [np.zeros(d, dtype=F32) for _ in range(n)]
    for rnd in range(2):
        grads = make_grads(d, n, seed=70 + rnd, bf16=bf16)
        dg = [x.to(DEV) for x in grads]
        gn = [to_np32(x) for x in grads]
        M_ref = o.prepare_range(P, gn, efs_ref)
        R.prepare(dg)
        R.compress_each(rnd, dg, range_M=torch.from_numpy(M_ref).to(DEV))
        pks = []
        for i in range(n):
            pk, ne = o.compress(P, i, rnd, gn[i], efs_ref[i], M_ref)
            assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"round {rnd} worker {i}")
            assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5, f"round {rnd} worker {i}"
            efs_ref[i] = ne
            R.efs[i].copy_(torch.from_numpy(ne))
            R.packed[i].copy_(torch.from_numpy(pk))
            pks.append(pk)
        R.aggregate()
        R.decompress(rnd, range_M=torch.from_numpy(M_ref).to(DEV))
        ref = o.decompress(P, rnd, o.aggregate(P, pks), M_ref)
        assert rel_l2(R.out.cpu().numpy(), ref) <= 1e-5


def test_bf16_gradients_with_error_feedback():
    block, K, n = 1 << 13, 2, 2
    d = block * K
    P, L = both_params(d, block, n, bf16=True)
    grads = make_grads(d, n, seed=5, bf16=True)
    R = GpuRound(L, ef=True)
    for e in R.efs:
        e.copy_(torch.randn(d, device=DEV) * 1e-4)
    efs0 = [e.cpu().numpy() for e in R.efs]
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    M_ref = o.prepare_range(P, gn, efs0)
    R.prepare(dg)
    assert np.all(np.abs(R.range_M.cpu().numpy() - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    R.compress_each(1, dg, range_M=torch.from_numpy(M_ref).to(DEV))
    for i in range(n):
        pk, ne = o.compress(P, i, 1, gn[i], efs0[i], M_ref)
        assert_indices_match(R.packed[i].cpu().numpy(), pk, 4)
        assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5


@pytest.mark.parametrize("L", [21, 23])
def test_blocks_that_need_a_middle_pass(L):
    """B > 2^20: bits above the first 13 are split over an in-place middle pass and the final pass."""
    block, n = 1 << L, 1
    P, Lp = both_params(block, block, n)
    grads = make_grads(block, n, seed=L)
    R = GpuRound(Lp, ef=True)
    dg = [x.to(DEV) for x in grads]
    R.prepare(dg)
    gn = [to_np32(x) for x in grads]
    M_ref = o.prepare_range(P, gn, [np.zeros(block, dtype=F32)])
    R.compress_each(0, dg, range_M=torch.from_numpy(M_ref).to(DEV))
    pk, ne = o.compress(P, 0, 0, gn[0], np.zeros(block, dtype=F32), M_ref)
    assert_indices_match(R.packed[0].cpu().numpy(), pk, 4)
    assert rel_l2(R.efs[0].cpu().numpy(), ne) <= 1e-5
    R.aggregate()
    R.decompress(0, range_M=torch.from_numpy(M_ref).to(DEV))
    ref = o.decompress(P, 0, o.aggregate(P, [pk]), M_ref)
    assert rel_l2(R.out.cpu().numpy(), ref) <= 1e-5


@pytest.mark.parametrize("order", [1, 0], ids=["split-order", "ascending-order"])
def test_largest_block_against_closed_forms(order):
    """B = 2^27, the largest block the library takes (13 + 7 + 7 bits).  The oracle needs minutes there, so the
    inputs are chosen to make every butterfly exact in any order: two nonzero coordinates going in
    (RHT(x)[j] = c (s1 h(j,k1) + 2 s2 h(j,k2)), h(j,k) = (-1)^popcount(j & k)), and sums that follow one Hadamard
    column coming back (the inverse is nonzero at coordinates 0 and k1 only).  The quantizer is the oracle's, on
    sampled tiles."""
    Lg = 27
    B = 1 << Lg
    k1, k2 = 0x2B5A6C9, 0x5D3C0F2
    P, Lp = both_params(B, B, 1, order=order)
    R = GpuRound(Lp)
    x = torch.zeros(B, dtype=torch.float32, device=DEV)
    x[k1], x[k2] = 1.0, 2.0
    R.prepare([x])
    xn = np.zeros(B, dtype=F32)
    xn[k1], xn[k2] = 1.0, 2.0
    M_ref = o.prepare_range(P, [xn])
    assert abs(float(R.range_M.cpu()[0]) - float(M_ref[0])) <= 2.0 ** -23 * float(M_ref[0])
    R.compress_each(3, [x], range_M=torch.from_numpy(M_ref).to(DEV))
    packed = R.packed[0].cpu().numpy()
    s1 = float(o.rademacher_signs(P.seed, 3, k1, 1)[0])
    s2 = float(o.rademacher_signs(P.seed, 3, k2, 1)[0])
    c = o.rht_scale(B)

    def h(j, k):
        v = j & k
        for sh in (16, 8, 4, 2, 1):
            v = v ^ (v >> sh)
        return 1 - 2 * (v & 1)

    T = 8192
    Pt = o.Params(d=T, block=T, n=1, b=P.b, g=P.g, t_p=P.t_p, seed=P.seed, table=P.table, agg_bits=8, order=order)
    rng = np.random.default_rng(27)
    tiles = [0, B // T - 1] + [int(t) for t in rng.integers(0, B // T, size=30)]
    for t in tiles:
        j = np.arange(t * T, (t + 1) * T, dtype=np.int64)
        Rt = ((s1 * h(j, k1) + 2.0 * s2 * h(j, k2)).astype(F32) * c).astype(F32)
        z = o.quantize_rotated(Pt, Rt, M_ref, o.sq_halfwords(P.seed, 3, 0, t * T, T))
        assert np.array_equal(packed[t * T // 2:(t + 1) * T // 2], o.pack_indices(z, P.b)), f"tile {t}"

    # decompression: Y = 20 where h(j, k1) = +1 and 10 where it is -1
    j = torch.arange(B, dtype=torch.int64, device=DEV)
    R.agg.copy_((15 + 5 * h(j, k1)).to(torch.uint8))
    del j
    R.decompress(3, range_M=torch.from_numpy(M_ref).to(DEV))
    _, _, step_n = o.block_scalars(P, M_ref)
    a = F32(F32(F32(20.0) * step_n[0]) - M_ref[0])
    b = F32(F32(F32(10.0) * step_n[0]) - M_ref[0])
    half = F32(2.0 ** (Lg - 1))
    sg0 = o.rademacher_signs(P.seed, 3, 0, 1)[0]
    want0 = F32(F32(F32(a + b) * half) * c) * sg0
    want1 = F32(F32(F32(a - b) * half) * c) * F32(s1)
    out = R.out
    assert float(out[0].cpu()) == float(want0) and float(out[k1].cpu()) == float(want1)
    assert int(torch.count_nonzero(out).cpu()) == 2


def test_a_round_captured_in_a_hip_graph_replays_bit_for_bit():
    """The four calls only launch kernels on the caller's stream (no allocation, no memset, no host sync), so a
    whole round can be captured once and replayed; every replay must equal the eager result, also after other
    eager work and synchronizations in between."""
    block, K, n = 1 << 16, 3, 4
    d = block * K
    _, L = both_params(d, block, n, order=1)
    grads = [x.to(DEV) for x in make_grads(d, n, seed=5)]
    E = GpuRound(L, ef=True)
    E.prepare(grads)
    E.compress_all(4, grads)
    E.aggregate()
    E.decompress(4)
    torch.cuda.synchronize()
    want = [t.clone() for t in (E.range_M, E.agg, E.out, *E.packed, *E.efs)]

    G = GpuRound(L, ef=True)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        G.prepare(grads)                       # warm-up on the capture stream
        torch.cuda.synchronize()
        for e in G.efs:
            e.zero_()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            G.prepare(grads)
            G.compress_all(4, grads)
            G.aggregate()
            G.decompress(4)
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        for e in G.efs:
            e.zero_()                             # the round updates the error-feedback buffers in place
        for t in (G.range_M, G.agg, G.out, *G.packed):
            t.fill_(0)
        scratch = torch.randn(1 << 20, device=DEV).sum()   # unrelated eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [G.range_M, G.agg, G.out, *G.packed, *G.efs]
        for a, b in zip(got, want):
            assert torch.equal(a, b), f"replay {rep}"
        del scratch


def test_homomorphism_on_the_library_itself():
    """Sec. 4.3's defining property, on the GPU alone: decompressing the aggregate of all workers equals the average
    of what each worker's stream decompresses to on its own (same table, same range), up to binary32 rounding."""
    block, K, n = 1 << 16, 4, 8
    d = block * K
    _, L = both_params(d, block, n, order=1)
    grads = [x.to(DEV) for x in make_grads(d, n, seed=12)]
    R = GpuRound(L)
    R.prepare(grads)
    R.compress_all(9, grads)
    R.aggregate()
    R.decompress(9)
    together = R.out.double().cpu().numpy()
    _, L1 = both_params(d, block, 1, order=1)                 # one worker at a time: Y = T[Z_i], n = 1
    S = GpuRound(L1)
    mean = np.zeros(d, dtype=np.float64)
    for i in range(n):
        api.thc_aggregate(L1, [R.packed[i]], S.agg)
        api.thc_decompress(L1, 9, S.agg, R.range_M, S.out, S.ws)
        mean += S.out.double().cpu().numpy()
    mean /= n
    assert rel_l2(together, mean) <= 1e-6
    # and it estimates the true mean of the inputs.  Every worker's error is about 0.02 ||x_max||^2 (the table's cost
    # for the shared range), the workers here have norms 1 : 1.3 : ... : 3.1, so the mean's NMSE stays below
    # 0.02 * n * 3.1^2 / sum_i (1 + 0.3 i)^2 = 0.042
    true = np.mean([g.double().cpu().numpy() for g in grads], axis=0)
    assert 0.005 < o.nmse(true, together) < 0.045


# ----------------------------------------------------------------------------- the single-launch sweep
@pytest.mark.parametrize("L,K,n,ef,bf16,first_block", [(17, 6, 2, False, False, 0), (17, 5, 3, True, False, 0),
                                                       (18, 4, 1, True, True, 0), (19, 7, 2, False, True, 3),
                                                       (20, 4, 2, True, False, 1 << 13), (17, 9, 5, False, False, 0)])
def test_single_launch_sweep_matches_the_oracle(L, K, n, ef, bf16, first_block):
    """thc_params.single_launch with the split stage order, blocks of 2^17 and more, at least four blocks:
    thc_compress_all and thc_compress run all passes of all blocks in one launch (blocks follow each other through a
    ring of slots, workgroups wait on counters).  Range, packed bytes and error feedback must equal the oracle's and the launch-by-launch path's,
    and the status word must stay 0 (no wait timed out, no workgroup ran on an unexpected XCD)."""
    block = 1 << L
    d, j0 = block * K, first_block * block
    P, Lp = both_params(d, block, n, bf16=bf16, order=1, first_block=first_block, single_launch=1)
    R = GpuRound(Lp, ef=ef)
    grads = make_grads(d, n, seed=L + K, bf16=bf16)
    for x in grads:
        x[2 * block:3 * block] = 0                                # an all-zero block on the way
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    efs0 = [to_np32(torch.randn(d, generator=torch.Generator().manual_seed(i)) * 2e-4) for i in range(n)] if ef else None
    for rnd in (3, 4):
        if ef:
            for i in range(n):
                R.efs[i].copy_(torch.from_numpy(efs0[i]))
        M_ref = o.prepare_range(P, gn, efs0)
        R.compress_all(rnd, dg)
        assert R.status() == 0
        M_gpu = R.range_M.cpu().numpy()
        assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
        assert ef or M_gpu[2] == 0.0
        new_efs = []
        for i in range(n):
            pk, ne = o.compress(P, i, rnd, gn[i], None if efs0 is None else efs0[i], M_gpu, j0=j0)
            assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"round {rnd} worker {i}")
            if ef:
                assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5, f"round {rnd} worker {i}"
                new_efs.append(ne)
        all_packed = [t.clone() for t in R.packed]
        all_efs = [t.clone() for t in R.efs] if ef else None
        # one worker at a time (thc_compress, the oracle's range): the same bytes as the oracle with that range
        dM = torch.from_numpy(M_ref).to(DEV)
        if ef:
            for i in range(n):
                R.efs[i].copy_(torch.from_numpy(efs0[i]))
        R.compress_each(rnd, dg, range_M=dM)
        assert R.status() == 0
        for i in range(n):
            pk, ne = o.compress(P, i, rnd, gn[i], None if efs0 is None else efs0[i], M_ref, j0=j0)
            assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"round {rnd} worker {i} alone")
            if ef:
                assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5
        # and the launch-by-launch path, two blocks to a group: bit for bit
        _, Lg = both_params(d, block, n, bf16=bf16, order=1, first_block=first_block, group_log2=L + 1)
        G = GpuRound(Lg, ef=ef)
        if ef:
            for i in range(n):
                G.efs[i].copy_(torch.from_numpy(efs0[i]))
        G.compress_all(rnd, dg)
        assert torch.equal(G.range_M, torch.from_numpy(M_gpu).to(DEV))
        for i in range(n):
            assert torch.equal(G.packed[i], all_packed[i])
            if ef:
                assert torch.equal(G.efs[i], all_efs[i])
        if ef:
            efs0 = new_efs


# ----------------------------------------------------------------------------- slices of a longer vector
@pytest.mark.parametrize("first_block,block,K,n,ef,order", [(5, 1 << 12, 3, 2, True, 0), (1 << 25, 1 << 10, 4, 2, False, 0),
                                                            (3, 1 << 16, 2, 2, True, 1), (4000, 1 << 21, 1, 1, True, 1)])
def test_buffers_that_hold_a_slice_of_a_longer_vector(first_block, block, K, n, ef, order):
    """thc_params.first_block: the random streams are indexed by the coordinate's position in the whole vector
    (also beyond 2^32), so a shard computes what the whole-vector call computes for its blocks."""
    d, j0 = block * K, first_block * block
    P, L = both_params(d, block, n, order=order, first_block=first_block)
    R = GpuRound(L, ef=ef)
    grads = make_grads(d, n, seed=first_block % 1000)
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    efs_ref = None
    if ef:
        efs_ref = [to_np32(torch.randn(d, generator=torch.Generator().manual_seed(9 + i)) * 1e-4) for i in range(n)]
        for i in range(n):
            R.efs[i].copy_(torch.from_numpy(efs_ref[i]))
    M_ref = o.prepare_range(P, gn, efs_ref)
    R.prepare(dg)
    R.compress_each(7, dg, range_M=torch.from_numpy(M_ref).to(DEV))
    pks = []
    for i in range(n):
        pk, ne = o.compress(P, i, 7, gn[i], None if efs_ref is None else efs_ref[i], M_ref, j0=j0)
        assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"worker {i}")
        if ef:
            assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5
        R.packed[i].copy_(torch.from_numpy(pk))
        pks.append(pk)
    R.aggregate()
    R.decompress(7, range_M=torch.from_numpy(M_ref).to(DEV))
    assert rel_l2(R.out.cpu().numpy(), o.decompress(P, 7, o.aggregate(P, pks), M_ref, j0=j0)) <= 1e-5


def test_two_slices_reproduce_the_whole_vector_bit_for_bit():
    block, K, n, cut = 1 << 13, 6, 2, 2
    d = block * K
    _, Lw = both_params(d, block, n)
    grads = [x.to(DEV) for x in make_grads(d, n, seed=77)]
    ef0 = [(torch.randn(d, generator=torch.Generator().manual_seed(i)) * 1e-4).to(DEV) for i in range(n)]
    W = GpuRound(Lw, ef=True)
    for i in range(n):
        W.efs[i].copy_(ef0[i])
    W.prepare(grads)
    W.compress_all(2, grads)
    W.aggregate()
    W.decompress(2)
    for lo, hi in ((0, cut), (cut, K)):
        a, b = lo * block, hi * block
        _, Ls = both_params(b - a, block, n, first_block=lo)
        S = GpuRound(Ls, ef=True)
        for i in range(n):
            S.efs[i].copy_(ef0[i][a:b])
        gs = [g[a:b] for g in grads]
        S.prepare(gs)
        S.compress_all(2, gs)
        S.aggregate()
        S.decompress(2)
        assert torch.equal(S.range_M, W.range_M[lo:hi])
        for i in range(n):
            assert torch.equal(S.packed[i], W.packed[i][a // 2:b // 2])
            assert torch.equal(S.efs[i], W.efs[i][a:b])
        assert torch.equal(S.agg, W.agg[a:b]) and torch.equal(S.out, W.out[a:b])


def _random_configurations(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        L = int(rng.integers(10, 18))
        K = int(rng.integers(1, 5))
        n = int(rng.integers(1, 7))
        b = int(rng.integers(1, 9))
        g = int(rng.integers(2 ** b - 1, min(255, 4 * 2 ** b) + 1))
        need = int(np.ceil(np.log2(g * n + 1)))
        agg_bits = int(rng.choice([need, 8, 16, int(rng.integers(need, 17))]))
        agg_bits = max(agg_bits, need)
        out.append((L, K, n, b, g, agg_bits, bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), int(rng.integers(0, 2)),
                    int(rng.choice([0, 0, 7, 1 << 23]))))
    return out


@pytest.mark.parametrize("L,K,n,b,g,agg_bits,ef,bf16,order,first_block", _random_configurations(16, 20230208))
def test_seeded_random_configurations(L, K, n, b, g, agg_bits, ef, bf16, order, first_block):
    """Valid parameter combinations drawn from a fixed seed: block size, worker count, index and sum widths,
    granularity (with the oracle's optimal table for it), error feedback, bf16 input, stage order, slice offset."""
    block = 1 << L
    d, j0 = block * K, first_block * block
    P, Lp = both_params(d, block, n, b=b, g=g, agg_bits=agg_bits, bf16=bf16, order=order, first_block=first_block)
    R = GpuRound(Lp, ef=ef)
    grads = make_grads(d, n, seed=L * 100 + K, bf16=bf16)
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    efs_ref = None
    if ef:
        efs_ref = [to_np32(torch.randn(d, generator=torch.Generator().manual_seed(i)) * 2e-4) for i in range(n)]
        for i in range(n):
            R.efs[i].copy_(torch.from_numpy(efs_ref[i]))
    M_ref = o.prepare_range(P, gn, efs_ref)
    R.prepare(dg)
    assert np.all(np.abs(R.range_M.cpu().numpy() - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    R.compress_each(5, dg, range_M=torch.from_numpy(M_ref).to(DEV))
    pks = []
    for i in range(n):
        pk, ne = o.compress(P, i, 5, gn[i], None if efs_ref is None else efs_ref[i], M_ref, j0=j0)
        assert_indices_match(R.packed[i].cpu().numpy(), pk, b, f"worker {i}")
        if ef:
            assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5
        R.packed[i].copy_(torch.from_numpy(pk))
        pks.append(pk)
    R.aggregate()
    Y = o.aggregate(P, pks)
    assert np.array_equal(R.agg.cpu().numpy(), o.aggregate_stream(P, Y))
    R.decompress(5, range_M=torch.from_numpy(M_ref).to(DEV))
    assert rel_l2(R.out.cpu().numpy(), o.decompress(P, 5, Y, M_ref, j0=j0)) <= 1e-5


# ----------------------------------------------------------------------------- degenerate cases
def test_all_zero_block_and_zero_padding():
    block, K, n = 1 << 12, 3, 2
    d = block * K
    P, L = both_params(d, block, n)
    grads = make_grads(d, n, seed=3)
    for x in grads:
        x[block:2 * block] = 0                   # an all-zero block: M = 0, every index 0, decodes to 0
        x[2 * block + 100:] = 0                  # a partly padded block
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    R.compress_all(0, dg)
    R.aggregate()
    R.decompress(0)
    M_ref = o.prepare_range(P, gn)
    M_gpu = R.range_M.cpu().numpy()
    assert M_gpu[1] == 0.0 and M_ref[1] == 0.0
    assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    for i in range(n):
        pk = R.packed[i].cpu().numpy()
        assert np.all(pk[block // 2: block] == 0)
    got = R.out.cpu().numpy()
    assert np.all(got[block:2 * block] == 0)
    packed = [o.compress(P, i, 0, gn[i], None, M_gpu)[0] for i in range(n)]
    for i in range(n):
        assert_indices_match(R.packed[i].cpu().numpy(), packed[i], 4)
    assert rel_l2(got, o.decompress(P, 0, o.aggregate(P, packed), M_gpu)) <= 1e-5


@pytest.mark.parametrize("L,order", [(12, 0), (13, 0), (16, 1), (17, 1)])
@pytest.mark.parametrize("k", [-80, 40, -100, -110, -115, -116, -120])
def test_very_small_and_very_large_magnitudes(L, order, k):
    """Inputs scaled by 2^k: the indices must equal the oracle's at every magnitude binary32 can hold.  M is about
    2.8e-3 * 2^k here.  Down to k = -115 the scale g / (M - m) is a finite binary32 number (from about k = -97 on the
    kernels leave their 2^16-scaled fast form for the plain one); at k = -116 it overflows and the block counts as
    empty on both sides; at k = -120 the inputs themselves are subnormal."""
    block, K, n = 1 << L, 2, 2
    d = block * K
    P, Lp = both_params(d, block, n, order=order)
    grads = [g * (2.0 ** k) for g in make_grads(d, n, seed=L)]
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    R = GpuRound(Lp)
    R.prepare(dg)
    M_ref = o.prepare_range(P, gn)
    assert np.all(np.abs(R.range_M.cpu().numpy() - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    Md = torch.from_numpy(M_ref).to(DEV)
    R.compress_each(1, dg, range_M=Md)
    pks = [o.compress(P, i, 1, gn[i], None, M_ref)[0] for i in range(n)]
    for i in range(n):
        assert np.array_equal(R.packed[i].cpu().numpy(), pks[i]), f"worker {i}"
    if k <= -116:
        assert all(not pk.any() for pk in pks)
    else:
        assert all(pk.any() for pk in pks)
    R.aggregate()
    R.decompress(1, range_M=Md)
    assert rel_l2(R.out.cpu().numpy(), o.decompress(P, 1, o.aggregate(P, pks), M_ref)) <= 1e-5


def test_truncation_is_taken_like_the_oracle():
    """Rotated coordinates beyond +-M are truncated (Alg. 3): for the worker with the largest norm about a
    p/2 fraction lands on the first and on the last index; an explicitly narrow range clamps far more."""
    block, n = 1 << 14, 2
    P, L = both_params(block, block, n)
    grads = make_grads(block, n, seed=11)
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    M_ref = o.prepare_range(P, [to_np32(x) for x in grads])
    for M in (M_ref, (M_ref * F32(0.25)).astype(F32)):
        R.prepare(dg)
        R.compress_each(6, dg, range_M=torch.from_numpy(M).to(DEV))
        for i in range(n):
            ref, _ = o.compress(P, i, 6, to_np32(grads[i]), None, M)
            assert_indices_match(R.packed[i].cpu().numpy(), ref, 4)
        z = o.unpack_indices(ref, 4)                 # the last worker has the largest norm
        lo_frac, hi_frac = (z == 0).mean(), (z == 15).mean()
        if M is M_ref:
            assert 0.005 < lo_frac < 0.04 and 0.005 < hi_frac < 0.04
        else:
            assert lo_frac > 0.25 and hi_frac > 0.25


def test_caller_supplied_range_without_thc_prepare_range():
    block, n = 1 << 13, 2
    P, L = both_params(2 * block, block, n)
    grads = make_grads(2 * block, n, seed=13)
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    M = np.array([3e-3, 5e-3], dtype=F32)
    R.compress_each(0, dg, range_M=torch.from_numpy(M).to(DEV))
    for i in range(n):
        ref, _ = o.compress(P, i, 0, to_np32(grads[i]), None, M)
        assert_indices_match(R.packed[i].cpu().numpy(), ref, 4)


def test_rounds_and_workers_use_different_random_streams_and_calls_are_deterministic():
    block, n = 1 << 13, 2
    P, L = both_params(block, block, n)
    g = make_grads(block, 1, seed=17)[0]
    grads = [g, g.clone()]                       # identical gradients on both workers
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    R.prepare(dg)
    R.compress_all(0, dg)
    a0, a1 = R.packed[0].cpu().numpy().copy(), R.packed[1].cpu().numpy().copy()
    assert not np.array_equal(a0, a1)            # independent rounding per worker (App. A)
    R.prepare(dg)
    R.compress_all(0, dg)
    assert np.array_equal(R.packed[0].cpu().numpy(), a0)      # same inputs, same bytes
    R.prepare(dg)
    R.compress_all(1, dg)
    assert not np.array_equal(R.packed[0].cpu().numpy(), a0)  # D^r and the draws change with the round


# ----------------------------------------------------------------------------- the bench configurations
def checksum64(t):
    """Sum of the buffer's 64-bit words modulo 2^64 (torch tensor or numpy array of bytes)."""
    if isinstance(t, np.ndarray):
        return int(np.frombuffer(t.tobytes(), dtype=np.uint64).sum(dtype=np.uint64))
    return int(t.view(torch.int64).sum().cpu()) & 0xFFFFFFFFFFFFFFFF


def _launch_shape_parity(w, blocks, workers=None, rounds=1, order=1, alone=None, single_launch=0):
    """A workload at the size and in the launch configuration bench.py times it in (thc_compress_all, thc_aggregate,
    thc_decompress on the whole vectors).  The oracle checks the sampled blocks (blocks are independent THC
    instances) for the sampled workers, working from the very range the GPU used, which itself must be within 2^-23
    of the oracle's.  Properties cover the rest: sums never exceed g*n, all-zero blocks decode to exact zeros.
    `alone`: a worker that is also compressed on its own (thc_compress) with the oracle's range for the sampled
    blocks."""
    workers = list(range(w.n)) if workers is None else workers
    T = o.solve_table(w.b, w.g, w.p)
    tp = o.t_p_of(w.p)
    B = w.block
    P_blk = o.Params(d=B, block=B, n=w.n, b=w.b, g=w.g, t_p=tp, seed=SEED, table=T, agg_bits=w.agg_bits, order=order)
    L = api.make_params(w.d, B, w.n, w.b, w.g, tp, SEED, T, w.agg_bits,
                        api.THC_DTYPE_BF16 if w.dtype == "bf16" else api.THC_DTYPE_F32, order, 0, 0, single_launch)
    grads = [wl.gradient(w, i, device=DEV) for i in range(w.n)]
    for i in (0, w.n - 1):
        print(f"{w.name} input {i}: {wl.checksum(grads[i][:1 << 24])}")
    R = GpuRound(L, ef=w.ef)
    compared = 0
    for rnd in range(rounds):
        ef_before = {(k, i): R.efs[i][k * B:(k + 1) * B].cpu().numpy() for k in blocks for i in range(w.n)} if w.ef else {}
        R.compress_all(rnd, grads)
        assert R.status() == 0
        R.aggregate()
        R.decompress(rnd)
        torch.cuda.synchronize()
        M_gpu = R.range_M.cpu().numpy()
        assert int(R.agg.view(torch.uint8 if w.agg_bits == 8 else torch.int16).max()) <= w.g * w.n
        print(f"{w.name} round {rnd}: packed checksums {[hex(checksum64(t)) for t in R.packed]}, sums {hex(checksum64(R.agg))}")
        for k in blocks:
            sl = slice(k * B, (k + 1) * B)
            gn = [to_np32(g[sl]) for g in grads]
            efs0 = [ef_before[(k, i)] for i in range(w.n)] if w.ef else None
            M_ref = o.prepare_range(P_blk, gn, efs0)
            assert abs(M_gpu[k] - M_ref[0]) <= abs(M_ref[0]) * 2.0 ** -23, f"block {k}"
            Mk = M_gpu[k:k + 1]
            for i in workers:
                pk, ne = o.compress(P_blk, i, rnd, gn[i], None if efs0 is None else efs0[i], Mk, j0=k * B)
                got = R.packed[i][k * B * w.b // 8:(k + 1) * B * w.b // 8].cpu().numpy()
                assert_indices_match(got, pk, w.b, f"{w.name} round {rnd} block {k} worker {i}")
                if w.ef:
                    assert rel_l2(R.efs[i][sl].cpu().numpy(), ne) <= 1e-5, f"block {k} worker {i}"
            # the sums of ALL workers' streams as the GPU wrote them, then the estimate from those sums
            Y = o.aggregate(P_blk, [t[k * B * w.b // 8:(k + 1) * B * w.b // 8].cpu().numpy() for t in R.packed])
            agg_k = R.agg[k * B * w.agg_bits // 8:(k + 1) * B * w.agg_bits // 8].cpu().numpy()
            assert np.array_equal(agg_k, o.aggregate_stream(P_blk, Y)), f"block {k}"
            assert checksum64(agg_k) == checksum64(o.aggregate_stream(P_blk, Y))
            ref = o.decompress(P_blk, rnd, Y, Mk, j0=k * B)
            assert rel_l2(R.out[sl].cpu().numpy(), ref) <= 1e-5, f"block {k}"
            compared += 1
        if alone is not None and not w.ef:
            # one worker on its own, the oracle's range injected for the sampled blocks
            rm = R.range_M.clone()
            refs = {}
            for k in blocks:
                gn = [to_np32(g[k * B:(k + 1) * B]) for g in grads]
                refs[k] = o.prepare_range(P_blk, gn)
                rm[k] = float(refs[k][0])
            pk_all = torch.zeros_like(R.packed[alone])
            api.thc_compress(L, alone, rnd, grads[alone], None, rm, pk_all, R.ws)
            assert R.status() == 0
            for k in blocks:
                pk, _ = o.compress(P_blk, alone, rnd, to_np32(grads[alone][k * B:(k + 1) * B]), None, refs[k], j0=k * B)
                assert_indices_match(pk_all[k * B * w.b // 8:(k + 1) * B * w.b // 8].cpu().numpy(), pk, w.b, f"alone, block {k}")
    assert compared == rounds * len(blocks)
    return R, grads


def _need_memory(gib):
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    if free < gib * (1 << 30):
        pytest.skip(f"needs about {gib} GiB of device memory")


@pytest.mark.timeout(900)
@pytest.mark.parametrize("order,single", [(1, 0), (0, 0), (1, 1)], ids=["split-order", "ascending-order", "single-launch"])
def test_vgg16_shape_full_size_sampled_blocks(order, single):
    """The 138M-coordinate / 2^28-padded, 8-worker, b=4 configuration (bench.py's default: the split order, launch by
    launch; bench.py --single-launch is the third case)."""
    w = wl.C3
    _need_memory(16)
    first_pad = (w.real + w.block - 1) // w.block          # blocks from here on are all zero
    blocks = (0, 14, 63, 131, first_pad - 1)               # conv part, FC part, the partly padded block
    R, _ = _launch_shape_parity(w, blocks, order=order, alone=5 if order == 1 else None, single_launch=single)
    M_gpu = R.range_M.cpu().numpy()
    assert np.all(M_gpu[first_pad:] == 0) and np.all(M_gpu[:first_pad] > 0)
    assert float(R.out[first_pad * w.block:].abs().max()) == 0.0
    assert all(int(t[first_pad * w.block // 2:].max()) == 0 for t in R.packed)


@pytest.mark.timeout(900)
def test_resnet50_shape_full_size_all_workers_two_rounds():
    """One 2^25-point transform over the zero-padded vector, 8 workers, error feedback carried into a second round
    (launch by launch: the block needs a middle pass).  The oracle transforms three of the eight workers."""
    _need_memory(8)
    _launch_shape_parity(wl.C2, (0,), workers=[0, 3, 7], rounds=2)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("w", [wl.C4_B4, wl.C4_B2], ids=lambda w: w.name)
def test_bert_large_shape_full_size_sampled_blocks(w):
    """321 blocks of 2^20 (not a multiple of the 64-tile spans the first pass permutes over), 16 workers; 16-bit
    sums at b = 4, 8-bit sums at b = 2."""
    _need_memory(40)
    _launch_shape_parity(w, (0, 63, 64, 320))


@pytest.mark.timeout(900)
@pytest.mark.parametrize("single", [0, 1], ids=["launch-by-launch", "single-launch"])
def test_gpt2_xl_shape_prefix_all_workers(single):
    """The first 48 blocks of 2^22 of the GPT-2-XL-shaped workload (what bench.py --workload c5_gpt2_xl --blocks 48
    runs): 32 workers, bf16 gradients, error feedback, two rounds; the oracle follows three workers."""
    _need_memory(70)
    _launch_shape_parity(wl.shrink(wl.C5, 48), (0, 47), workers=[0, 13, 31], rounds=2, single_launch=single)


@pytest.mark.timeout(1500)
def test_gpt2_xl_shape_full_length_24_workers():
    """The GPT-2-XL-shaped workload at its full length (1,557,611,200 coordinates, 372 blocks of 2^22, bf16, error
    feedback).  With the 32 workers the configuration names, the buffers alone take 334 GB, more than the GPU has; 24
    workers (255 GB with a 2 GB workspace) are what fits, and the length is never cut.  Two rounds; the oracle follows
    two workers on three blocks, the last one partly padding."""
    _need_memory(262)
    w = wl.replace(wl.C5, n=24, name="c5_gpt2_xl_n24")
    _launch_shape_parity(w, (0, 200, 371), workers=[0, 23], rounds=2)


# ----------------------------------------------------------------------------- the other workload recipes
def _round_vs_oracle(w, rnd=1, rounds=1):
    """Whole rounds of a (shrunk) workload on the GPU against the oracle; the oracle's range is injected."""
    T = o.solve_table(w.b, w.g, w.p)
    tp = o.t_p_of(w.p)
    P = o.Params(d=w.d, block=w.block, n=w.n, b=w.b, g=w.g, t_p=tp, seed=SEED, table=T, agg_bits=w.agg_bits)
    L = api.make_params(w.d, w.block, w.n, w.b, w.g, tp, SEED, T, w.agg_bits,
                        api.THC_DTYPE_BF16 if w.dtype == "bf16" else api.THC_DTYPE_F32)
    grads = [wl.gradient(w, i, device=DEV) for i in range(w.n)]
    gn = [to_np32(g) for g in grads]
    R = GpuRound(L, ef=w.ef)
    efs_ref = [np.zeros(w.d, dtype=F32) for _ in range(w.n)] if w.ef else None
    for r in range(rnd, rnd + rounds):
        M_ref = o.prepare_range(P, gn, efs_ref)
        R.prepare(grads)
        M_gpu = R.range_M.cpu().numpy()
        assert np.all(np.abs(M_gpu - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
        dM = torch.from_numpy(M_ref).to(DEV)
        R.compress_each(r, grads, range_M=dM)
        packed_ref, new_efs = [], []
        for i in range(w.n):
            pk, ne = o.compress(P, i, r, gn[i], None if efs_ref is None else efs_ref[i], M_ref)
            assert_indices_match(R.packed[i].cpu().numpy(), pk, w.b, f"{w.name} round {r} worker {i}")
            packed_ref.append(pk)
            if w.ef:
                assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5
                new_efs.append(ne)
        R.aggregate()
        Y = o.aggregate(P, packed_ref)
        assert np.mean(R.agg_numpy() != Y) <= 1e-6 * w.n
        R.decompress(r, range_M=dM)
        assert rel_l2(R.out.cpu().numpy(), o.decompress(P, r, Y, M_ref)) <= 1e-5
        if w.ef:
            efs_ref = new_efs
            for i in range(w.n):
                R.efs[i].copy_(torch.from_numpy(efs_ref[i]))


def test_workload_c1_full():
    _round_vs_oracle(wl.C1)                                  # d = 2^20, n = 4: the whole configuration


def test_workload_c2_shape_single_transform_with_error_feedback():
    # ResNet-50 shape: one 2^25-point transform over the zero-padded vector, Laplace segments, error feedback,
    # two rounds so that the second one reads a real error buffer.  Two of the eight workers.
    _round_vs_oracle(wl.shrink(wl.C2, 1, n=2), rnd=0, rounds=2)


@pytest.mark.parametrize("w", [wl.C4_B4, wl.C4_B2], ids=lambda w: w.name)
def test_workload_c4_shape_first_blocks(w):
    # BERT-large shape: 16 workers with different sigmas and 50-sigma outliers; b = 4 -> 16-bit sums, b = 2 -> 8-bit
    _round_vs_oracle(wl.shrink(w, 2))


def test_workload_c5_shape_first_block():
    # GPT-2-XL shape: bf16 gradients, Student-t tails, 2^22 blocks, error feedback; 3 of the 32 workers
    _round_vs_oracle(wl.shrink(wl.C5, 1, n=3), rnd=0, rounds=2)


# ----------------------------------------------------------------------------- partial aggregation (Sec. 6)
def test_partial_aggregation_with_exact_width_sums():
    """The PS may aggregate only the workers that answered in time (Sec. 6; 90 % suffices in Sec. 8.4): the sum runs over a
    subset, the workers divide by its size, and ceil(log2(g m + 1)) bits per sum are enough (Sec. 8.4)."""
    import math
    block, K, n = 1 << 13, 3, 8
    d = block * K
    P, L = both_params(d, block, n)
    grads = make_grads(d, n, seed=23)
    R = GpuRound(L)
    dg = [x.to(DEV) for x in grads]
    R.prepare(dg)
    R.compress_all(7, dg)
    M = R.range_M.cpu().numpy()
    subset = [0, 2, 3, 5, 6, 7]                                   # two stragglers left out
    m = len(subset)
    w = math.ceil(math.log2(30 * m + 1))                          # 8 bits for 181 values
    Pm, Lm = both_params(d, block, m, agg_bits=w)
    agg = torch.zeros(d * w // 8, dtype=torch.uint8, device=DEV)
    out = torch.zeros(d, dtype=torch.float32, device=DEV)
    api.thc_aggregate(Lm, [R.packed[i] for i in subset], agg)
    Y = o.aggregate(Pm, [R.packed[i].cpu().numpy() for i in subset])
    assert np.array_equal(agg.cpu().numpy(), o.aggregate_stream(Pm, Y))
    api.thc_decompress(Lm, 7, agg, R.range_M, out, R.ws)
    ref = o.decompress(Pm, 7, Y, M)
    assert rel_l2(out.cpu().numpy(), ref) <= 1e-5
    # the estimate is of the subset's mean (the range of all eight workers still bounds it)
    mean_sub = np.mean([to_np32(grads[i]).astype(np.float64) for i in subset], axis=0)
    assert o.nmse(mean_sub, out.cpu().numpy()) < 0.03
    # a narrower sum: 4 of 8 workers need only 7 bits
    P4, L4 = both_params(d, block, 4, agg_bits=7)
    agg7 = torch.zeros(d * 7 // 8, dtype=torch.uint8, device=DEV)
    api.thc_aggregate(L4, R.packed[:4], agg7)
    Y4 = o.aggregate(P4, [R.packed[i].cpu().numpy() for i in range(4)])
    assert np.array_equal(agg7.cpu().numpy(), o.aggregate_stream(P4, Y4))
    api.thc_decompress(L4, 7, agg7, R.range_M, out, R.ws)
    assert rel_l2(out.cpu().numpy(), o.decompress(P4, 7, Y4, M)) <= 1e-5


# ----------------------------------------------------------------------------- the split stage order
@pytest.mark.parametrize("L,K,n,ef", [(16, 3, 2, False), (17, 2, 2, True), (18, 1, 3, False), (20, 2, 4, True), (21, 1, 1, True),
                                      (22, 1, 2, False), (23, 1, 1, True), (15, 2, 2, True)])
def test_split_stage_order(L, K, n, ef):
    """THC_ORDER_SPLIT: bits 0..9, 13..15, then 10..12, 16..: the first pass works on eight rows of 1024 coordinates.
    Same checks as for the ascending order, against the oracle running the same order."""
    block = 1 << L
    d = block * K
    P, Lp = both_params(d, block, n, order=1)
    grads = make_grads(d, n, seed=L * 7 + K)
    R = GpuRound(Lp, ef=ef)
    dg = [x.to(DEV) for x in grads]
    gn = [to_np32(x) for x in grads]
    efs0 = [np.zeros(d, dtype=F32) for _ in range(n)] if ef else None
    M_ref = o.prepare_range(P, gn, efs0)
    R.prepare(dg)
    assert np.all(np.abs(R.range_M.cpu().numpy() - M_ref) <= np.abs(M_ref) * 2.0 ** -23)
    dM = torch.from_numpy(M_ref).to(DEV)
    R.compress_each(2, dg, range_M=dM)
    packed_ref = []
    for i in range(n):
        pk, ne = o.compress(P, i, 2, gn[i], None if efs0 is None else efs0[i], M_ref)
        assert_indices_match(R.packed[i].cpu().numpy(), pk, 4, f"worker {i}")
        packed_ref.append(pk)
        if ef:
            assert rel_l2(R.efs[i].cpu().numpy(), ne) <= 1e-5
    R.aggregate()
    Y = o.aggregate(P, packed_ref)
    assert np.array_equal(R.agg_numpy(), Y)
    R.decompress(2, range_M=dM)
    ref = o.decompress(P, 2, Y, M_ref)
    assert np.array_equal(R.out.cpu().numpy(), ref)
