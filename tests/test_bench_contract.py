"""Host-side checks of bench.py and of the byte models its figures rest on (no GPU)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)

import bench  # noqa: E402
from paper_2302_08545_amd import workloads as wl  # noqa: E402


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""


@pytest.mark.parametrize("w,want", [(wl.C1, 26.0), (wl.C2, 110.0), (wl.C3, 46.0), (wl.C4_B4, 88.0), (wl.C4_B2, 78.0),
                                    (wl.C5, 360.0)], ids=lambda x: getattr(x, "name", str(x)))
def test_compulsory_bytes_per_coordinate(w, want):
    # every datum once: n (in + [EF 4 + 4] + b/8) + (n b/8 + w/8) + (w/8 + 4), written out per workload by hand
    assert wl.bytes_per_coord(w) == want


@pytest.mark.parametrize("w,want", [(wl.C3, 8 * 12.5 + 5 + 13), (wl.C4_B4, 16 * 12.5 + 10 + 14),
                                    (wl.C2, 8 * (12 + 8 + 4.5 + 4.5 + 8 + 16) + 5 + (1 + 4 + 8 + 8))],
                         ids=lambda x: getattr(x, "name", str(x)))
def test_moved_bytes_per_coordinate_of_the_pass_structure(w, want):
    # two passes (three for the 2^25 block), each reading and writing the vector once
    assert wl.moved_bytes_per_coord(w) == want


def test_counted_traffic_of_the_default_workload_is_read_from_the_tracked_profile():
    t = bench.measured_traffic("c3_vgg16")
    assert t is not None
    # the forward sweep moves 12.5 bytes per worker-coordinate through the L2s (and 16 MiB of partial sums)
    assert 0.99 < t / (8 * 2 ** 28 * 12.5) < 1.02
    assert bench.measured_traffic("no_such_workload") is None


def test_the_largest_kernel_of_the_default_workload_is_read_from_the_tracked_profile():
    name, per_round, avg_us = bench.profiled_kernel("c3_vgg16", "k_fwd_lo")
    assert name.startswith("k_fwd_lo<13") and per_round == 4 and 500 < avg_us < 1000
    assert bench.profiled_kernel("no_such_workload", "k_fwd_lo") is None
