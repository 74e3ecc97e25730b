"""Host logic of the library, checked without a GPU: how a transform is cut into passes and how every pass
tiles a block (thc_describe_plan).  The tiling tables are what the kernels index memory with, so they are
emulated here and must touch every coordinate of a span exactly once; the stage order must be the oracle's."""
import numpy as np
import pytest

from oracle import thc_oracle as o
from paper_2302_08545_amd import api

TILE_LOG2 = 13


def _params(L, order, K=1):
    T = o.solve_table(4, 30, 1 / 32)
    return api.make_params((1 << L) * K, 1 << L, 2, 4, 30, 2.15, 7, T, 8, stage_order=order)


def _tile_base(rec, tile):
    tib = tile & ((1 << rec["nfixed"]) - 1)
    off = np.zeros_like(tile)
    for c, m, p in zip(rec["fcum"], rec["fmask"], rec["fpos"]):
        off |= ((tib >> c) & m) << p
    return ((tile >> rec["nfixed"]) << rec["L"]) | off


def _in_tile(rec, idx):
    if rec["kind"] == 0:
        return idx
    if rec["kind"] == 3:
        return (idx & 1023) | ((idx >> 10) << 13)
    row = idx >> rec["logw"]
    n0 = rec["n0"]
    return ((row & ((1 << n0) - 1)) << rec["sh0"]) | ((row >> n0) << rec["sh1"]) | (idx & ((1 << rec["logw"]) - 1))


def _bit_sets(rec):
    cols = set(range(rec["logw"]))
    if rec["kind"] == 0:
        rows = set()
    elif rec["kind"] == 3:
        rows = {13, 14, 15}
    else:
        n0, nr = rec["n0"], rec["nrows"]
        rows = {rec["sh0"] + i for i in range(n0)} | {rec["sh1"] + i for i in range(nr - n0)}
    fixed = set()
    for m, p in zip(rec["fmask"], rec["fpos"]):
        fixed |= {p + i for i in range(int(m).bit_length())}
    return cols, rows, fixed


@pytest.mark.parametrize("order", [0, 1])
@pytest.mark.parametrize("L", list(range(10, 28)))
def test_passes_follow_the_stage_order_and_partition_the_offset_bits(L, order):
    recs = api.thc_describe_plan(_params(L, order, K=1 if L >= 19 else 1 << (19 - L)))
    bits = [b for r in recs for b in r["bits"]]
    assert bits == o.stage_order(1 << L, order)
    assert recs[0]["kind"] in (0, 3) and recs[-1]["kind"] == 2 and all(r["kind"] == 1 for r in recs[1:-1])
    assert len(recs) == (2 if L - 13 <= 9 else 3)
    for r in recs:
        cols, rows, fixed = _bit_sets(r)
        span = max(r["L"], TILE_LOG2)
        assert not (cols & rows) and not (cols & fixed) and not (rows & fixed)
        assert cols | rows | fixed == set(range(span)), (r, cols, rows, fixed)
        assert len(cols) + len(rows) == TILE_LOG2 and len(fixed) == r["nfixed"]
        if r["kind"] in (1, 2):
            assert sorted(rows) == sorted(r["bits"])          # a strided pass owns exactly the bits it transforms
            assert 2 <= len(rows) <= 9 or L - 13 < 2
        # where the low three bits of the tile index (the XCD of the workgroup) land
        if r["nfixed"] >= 3 and r["fmask"][0] >= 7:
            xcd = r["fpos"][0]
            if r["kind"] == 3:
                assert xcd == 10
            elif r["kind"] == 0:
                assert xcd == 16
            else:
                assert xcd == (13 if recs[0]["kind"] == 3 else 10)


@pytest.mark.parametrize("L,order,K", [(10, 0, 512), (12, 0, 3), (13, 0, 64), (15, 0, 16), (16, 1, 8), (17, 1, 1), (18, 0, 2),
                                       (19, 1, 1), (20, 1, 1), (20, 0, 1), (21, 1, 1), (22, 0, 1), (22, 1, 1), (23, 1, 1)])
def test_every_pass_touches_every_coordinate_exactly_once(L, order, K):
    """Emulation of the kernels' addressing: tile base from the workgroup id, offset inside the tile from the
    thread's tile index."""
    p = _params(L, order, K)
    d = (1 << L) * K
    for r in api.thc_describe_plan(p):
        ntiles = (d + (1 << TILE_LOG2) - 1) >> TILE_LOG2
        tile = np.arange(ntiles, dtype=np.int64)[:, None]
        idx = np.arange(1 << TILE_LOG2, dtype=np.int64)[None, :]
        coord = (_tile_base(r, tile) + _in_tile(r, idx)).reshape(-1)
        coord = coord[coord < d]                      # the guard of a partial last tile
        assert coord.size == d
        seen = np.zeros(d, dtype=np.uint8)
        seen[coord] = 1
        assert seen.all(), (r["kind"], r["bits"])
        # a strided tile stays inside one block; a tile of the first pass too, when blocks are at least a tile
        if L >= TILE_LOG2:
            blocks = (_tile_base(r, tile) + _in_tile(r, idx)) >> L
            assert np.all(blocks == blocks[:, :1])
