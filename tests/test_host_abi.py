"""Host-side checks that need no GPU: the C-ABI library loads and exports what include/thc.h declares,
argument validation returns the documented codes before any device work, and the host helpers
(threshold, table solver) agree with the oracle's independent implementations."""
import math
import os
import re

import pytest
import scipy.stats

from oracle import thc_oracle as o
from paper_2302_08545_amd import api

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
T430 = [0, 3, 5, 7, 9, 11, 13, 14, 15, 17, 19, 21, 23, 25, 27, 30]


def _p(**kw):
    base = dict(d=1 << 12, block=1 << 10, n=4, b=4, g=30, t_p=2.1538746, seed=7, table=T430, agg_bits=8)
    base.update(kw)
    return api.make_params(**base)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "thc.h")).read()
    declared = set(re.findall(r"\b(thc_[a-z_]+)\s*\(", header))
    declared -= {"thc_status"}
    assert declared == set(api.EXPORTS)
    L = api.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert api.thc_version() >= 100
    assert api.thc_strerror(0) == "THC_OK" and api.thc_strerror(-2) == "THC_ETABLE"


def test_params_struct_layout_matches_header(tmp_path):
    # d, block (8+8) n b g agg_bits in_dtype t_p (6*4) seed (8) table (256) stage_order first_block group_log2
    # reserved (4*4) = 320 bytes
    import ctypes
    import shutil
    import subprocess
    assert ctypes.sizeof(api.thc_params) == 320
    assert api.thc_params.seed.offset == 40 and api.thc_params.table.offset == 48
    # the header is plain C: compile it with gcc and compare every field's offset with the binding's
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    fields = [f[0] for f in api.thc_params._fields_]
    src = tmp_path / "layout.c"
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "thc.h"\nint main(void) {\n'
                   + "".join(f'  printf("{f} %zu\\n", offsetof(thc_params, {f}));\n' for f in fields)
                   + '  printf("sizeof %zu\\n", sizeof(thc_params));\n  return 0;\n}\n')
    exe = tmp_path / "layout"
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                    str(exe)], check=True)
    out = dict(line.split() for line in subprocess.run([str(exe)], check=True, capture_output=True,
                                                       text=True).stdout.splitlines())
    for f in fields:
        assert int(out[f]) == getattr(api.thc_params, f).offset, f
    assert int(out["sizeof"]) == ctypes.sizeof(api.thc_params)


def test_workspace_size():
    p = _p()
    # a ring that holds one group of blocks of all n workers + one double per min(B, 8192) coordinates per worker
    assert api.thc_workspace_bytes(p) >= 4 * (1 << 12) * 4 + 4 * 4 * 8
    # it does not grow with d: the 2^28 vector of the VGG16-shaped workload takes a ring of 2^29 values (one group of
    # blocks of all workers), not n * d = 2^31
    big = _p(d=1 << 28, block=1 << 20, n=8)
    assert (1 << 29) * 4 <= api.thc_workspace_bytes(big) < (1 << 29) * 4 * 1.02
    assert api.thc_workspace_bytes(_p(d=1 << 30, block=1 << 20, n=8)) < (1 << 29) * 4 * 1.05
    small = _p(d=1 << 28, block=1 << 20, n=8, group_log2=22)
    assert api.thc_workspace_bytes(small) < api.thc_workspace_bytes(big) / 3
    # the single-launch sweep takes a ring of a few block-sized slots per worker: 4 without, 8 with error feedback
    # (two more phases follow each block), e.g. 32 workers with 2^22 blocks
    wide = dict(d=372 << 22, block=1 << 22, n=32, agg_bits=16, stage_order=1, single_launch=1, group_log2=0)
    no_ef, with_ef = api.thc_workspace_bytes(_p(**wide), False), api.thc_workspace_bytes(_p(**wide), True)
    assert 4 * 32 * (1 << 22) * 4 <= no_ef < 4 * 32 * (1 << 22) * 4 * 1.05
    assert 8 * 32 * (1 << 22) * 4 <= with_ef < 8 * 32 * (1 << 22) * 4 * 1.05
    sweep = _p(d=1 << 28, block=1 << 20, n=8, stage_order=1, single_launch=1)
    assert 4 * 8 * (1 << 20) * 4 <= api.thc_workspace_bytes(sweep) < api.thc_workspace_bytes(big)
    # the uniform variant with rotation keeps all n rotated vectors
    u = api.make_params(1 << 20, 1 << 12, 4, 4, 15, 2.0, 7, list(range(16)), 8)
    assert api.thc_uniform_workspace_bytes(u, True) >= 4 * (1 << 20) * 4
    assert api.thc_uniform_workspace_bytes(u, False) < (1 << 20)


@pytest.mark.parametrize("kw,code", [
    (dict(block=1000), -1),                    # not a power of two
    (dict(block=1 << 9, d=1 << 12), -1),       # below the supported range
    (dict(d=(1 << 12) + 1), -1),               # not a multiple of the block
    (dict(n=0), -1),
    (dict(n=65, agg_bits=16), -4),             # more workers than a launch can take
    (dict(b=0), -1),
    (dict(b=9), -1),
    (dict(g=14), -1),                          # g < 2^b - 1
    (dict(agg_bits=0), -1),
    (dict(agg_bits=17), -1),
    (dict(agg_bits=6), -3),                    # 30 * 4 = 120 needs 7 bits
    (dict(t_p=0.0), -1),
    (dict(table=[0, 3, 5, 7, 9, 11, 13, 13, 15, 17, 19, 21, 23, 25, 27, 30]), -2),   # not strictly increasing
    (dict(table=[1] + T430[1:]), -2),          # T[0] != 0
    (dict(table=T430[:-1] + [29]), -2),        # T[last] != g
    (dict(n=9), -3),                           # 30 * 9 = 270 > 255: the prototype's eight-worker limit (Sec. 8 setup)
    (dict(n=16, agg_bits=8), -3),
    (dict(d=1 << 40, block=1 << 20), -1),      # more tiles than a 32-bit grid index
    (dict(stage_order=2), -1),
    (dict(group_log2=9), -1),
    (dict(group_log2=41), -1),
    (dict(single_launch=2), -1),
])
def test_validation_codes(kw, code):
    p = _p(**kw)
    L = api.lib()
    import ctypes as C
    out = C.c_size_t(0)
    assert L.thc_workspace_bytes(C.byref(p), 0, C.byref(out)) == code
    # the compute entry points validate first and return the same code without touching the device
    assert L.thc_aggregate(C.byref(p), None, None, None) == code
    assert L.thc_decompress(C.byref(p), 0, None, None, None, None, None) == code
    assert L.thc_compress(C.byref(p), 0, 0, None, None, None, None, None, None) == code
    assert L.thc_prepare_range(C.byref(p), None, None, None, None, None) == code
    assert L.thc_compress_all(C.byref(p), 0, None, None, None, None, None, None) == code


def test_null_and_misaligned_pointers_are_rejected_on_the_host():
    import ctypes as C
    p = _p()
    L = api.lib()
    assert L.thc_aggregate(C.byref(p), None, None, None) == -1
    assert L.thc_decompress(C.byref(p), 0, None, None, None, None, None) == -1
    assert L.thc_decompress(C.byref(p), 0, 16, 16, 24, 16, None) == -1          # out not 16-byte aligned
    assert L.thc_compress(C.byref(p), 4, 0, None, None, 16, 16, 16, None) == -1  # worker id out of range
    assert L.thc_compress(C.byref(p), 0, 1 << 32, None, None, 16, 16, 16, None) == -1   # round must fit 32 bits
    arr = (C.c_void_p * 4)(16, 16, 16, 8)
    assert L.thc_prepare_range(C.byref(p), arr, None, 16, 16, None) == -1    # one misaligned gradient
    assert L.thc_prepare_range(C.byref(p), (C.c_void_p * 4)(16, 16, 16, 16), None, None, 16, None) == -1   # no range
    assert L.thc_compress(C.byref(p), 0, 0, None, None, 16, 16, 16, None) == -1   # no gradient
    pk = (C.c_void_p * 4)(16, 16, 16, 16)
    assert L.thc_compress_all(C.byref(p), 0, arr, None, 16, pk, 16, None) == -1   # one misaligned gradient
    assert L.thc_compress_all(C.byref(p), 0, pk, None, 16, (C.c_void_p * 4)(16, 16, 0, 16), 16, None) == -1
    assert L.thc_workspace_bytes(None, 0, None) == -1


def test_threshold_matches_definition():
    for p in (1 / 32, 1 / 512, 1 / 1024, 0.5, 1e-6):
        t = api.thc_threshold(p)
        assert t == pytest.approx(scipy.stats.norm.isf(p / 2), rel=1e-12)
        assert t == pytest.approx(o.t_p_of(p), rel=1e-12)
    assert math.isnan(api.thc_threshold(0.0)) and math.isnan(api.thc_threshold(1.5))
    import numpy as np
    assert np.float32(api.thc_threshold(1 / 32)) == np.float32(o.t_p_of(1 / 32))


@pytest.mark.parametrize("b,g,p", [(4, 30, 1 / 32), (2, 8, 1 / 32), (4, 15, 1 / 32), (4, 36, 1 / 32), (4, 20, 1 / 512),
                                   (4, 51, 1 / 32), (3, 12, 1 / 1024), (3, 21, 1 / 1024), (2, 4, 1 / 32), (1, 1, 1 / 32),
                                   (1, 9, 1 / 32), (4, 16, 1 / 32), (2, 3, 1 / 32), (3, 40, 1 / 1024)])
def test_table_solver_matches_oracle(b, g, p):
    table, cost = api.thc_solve_table(b, g, p)
    assert table == o.solve_table(b, g, p)
    assert cost == pytest.approx(o.table_cost(table, g, o.t_p_of(p)), rel=1e-10)


def test_table_solver_rejects_bad_arguments():
    import ctypes as C
    L = api.lib()
    out = (C.c_uint8 * 256)()
    assert L.thc_solve_table(4, 14, 1 / 32, out, None) == -1      # g < 2^b - 1
    assert L.thc_solve_table(0, 14, 1 / 32, out, None) == -1
    assert L.thc_solve_table(4, 300, 1 / 32, out, None) == -1
    assert L.thc_solve_table(4, 30, 0.0, out, None) == -1
    assert L.thc_solve_table(4, 30, 1 / 32, None, None) == -1


def test_workload_recipes_on_cpu():
    import torch
    from paper_2302_08545_amd import workloads as wl
    assert wl.C3.d == 1 << 28 and wl.C3.K == 256 and wl.C4_B4.d == 321 << 20 and wl.C5.d == 372 << 22
    assert wl.bytes_per_coord(wl.C3) == 46 and wl.bytes_per_coord(wl.C1) == 26
    assert wl.bytes_per_coord(wl.C2) == 110 and wl.bytes_per_coord(wl.C4_B4) == 88
    assert wl.bytes_per_coord(wl.C4_B2) == 78 and wl.bytes_per_coord(wl.C5) == 360
    seg = wl.resnet50_segments(wl.C2.real)
    assert len(seg) == 161 and sum(seg) == wl.C2.real
    small = wl.shrink(wl.C3, 2, n=2)
    g0 = wl.gradient(small, 0)
    g0b = wl.gradient(small, 0)
    g1 = wl.gradient(small, 1)
    assert g0.shape == (2 << 20,) and torch.equal(g0, g0b) and not torch.equal(g0, g1)
    assert abs(float(g0.std()) - 1e-3) < 2e-5
    c1 = wl.gradient(wl.C1, 3)
    assert c1.dtype == torch.float32 and abs(float(c1.std()) - 1e-3) < 2e-5
    c5 = wl.gradient(wl.shrink(wl.C5, 1, n=1), 0)
    assert c5.dtype == torch.bfloat16 and c5.shape == (1 << 22,)
    c4 = wl.gradient(wl.shrink(wl.C4_B2, 1, n=1), 0)
    sig = float(c4.abs().median()) / 0.6745
    assert 0.5e-4 < sig < 2e-2 and 0.0005 < float((c4.abs() > 40 * sig).float().mean()) < 0.002
    c2 = wl.gradient(wl.shrink(wl.C2, 1, n=1), 0)
    assert int((c2[wl.C2.real:] != 0).sum()) == 0 and int((c2[:wl.C2.real] != 0).sum()) > 0.99 * wl.C2.real


# ----------------------------------------------------------------------------- table tool (App. B)
@pytest.mark.parametrize("b,g", [(1, 1), (1, 7), (2, 3), (2, 4), (2, 9), (2, 16), (2, 30), (3, 7), (3, 8), (3, 13), (3, 18),
                                 (3, 21), (4, 15), (4, 16), (4, 19), (4, 22)])
def test_exhaustive_search_agrees_with_the_shortest_path_solver(b, g):
    for p in (1 / 32, 1 / 1024):
        tb, cb, cnt = api.thc_solve_table_bruteforce(b, g, p)
        td, cd = api.thc_solve_table(b, g, p)
        assert cnt == math.comb(g - 1, 2 ** b - 2)         # strictly increasing tables from 0 to g
        assert tb == td and cb == pytest.approx(cd, rel=1e-12)
        assert tb == o.solve_table(b, g, p)


def test_exhaustive_search_refuses_hopeless_sizes():
    import ctypes as C
    out = (C.c_uint8 * 256)()
    assert api.lib().thc_solve_table_bruteforce(4, 51, 1 / 32, out, None, None) == -4    # C(50, 14) ~ 9.4e11 candidates
    assert math.comb(50, 14) > 4e9


def test_all_tables_the_paper_mentions_within_seconds():
    import time
    from paper_2302_08545_amd import tables
    t0 = time.perf_counter()
    all_t = tables.solve_all()
    dt = time.perf_counter() - t0
    assert len(all_t) == sum(51 - (2 ** b - 1) + 1 for b in (1, 2, 3, 4)) * len(tables.P_VALUES)
    assert dt < 60                                         # App. B: thousands of tables "within mere minutes"
    for (b, g, p), (t, c) in all_t.items():
        assert t[0] == 0 and t[-1] == g and all(x < y for x, y in zip(t, t[1:]))
    # cost falls with the bit budget and, at fixed b, a grid that refines another is never worse
    for p in tables.P_VALUES:
        assert all_t[(2, 24, p)][1] > all_t[(3, 24, p)][1] > all_t[(4, 24, p)][1]
        for b in (2, 3, 4):
            for g in range(2 ** b - 1, 26):
                assert all_t[(b, 2 * g, p)][1] <= all_t[(b, g, p)][1] * (1 + 1e-12)
