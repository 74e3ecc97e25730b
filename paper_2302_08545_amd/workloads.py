"""Seeded synthetic gradients shaped like the paper's vision / language workloads.

These generators hold none of the method's arithmetic; they serve the tests (which feed the same
tensors to the HIP library and to the CPU oracle) and bench.py.  The paper trains VGG16 / ResNet50 on
ImageNet1K / CIFAR100 and language models on GLUE-SST2 (Sec. 8); those datasets are not available here,
so each workload is a random vector with the coordinate count, per-layer scale structure and tail
behaviour of the corresponding model's flattened gradient, zero-padded to a multiple of the RHT block.

Every generator is deterministic given (base seed, worker id, device type).  CPU and GPU generators
draw different streams, so a test always generates on one device and copies.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, replace
from typing import List, Optional

import torch

BASE_SEED = 20230208
RHT_SEED = 0x5448435F53454544


@dataclass(frozen=True)
class Workload:
    name: str
    real: int            # coordinates that carry data
    d: int               # padded length (multiple of block)
    block: int           # RHT block
    n: int               # workers
    b: int
    g: int
    agg_bits: int
    dtype: str           # "f32" or "bf16"
    ef: bool             # error feedback enabled
    kind: str            # which recipe below
    p: float = 1.0 / 32  # support parameter of the paper's default configuration (Sec. 8 setup)

    @property
    def K(self) -> int:
        return self.d // self.block


def _pad(real: int, block: int) -> int:
    return (real + block - 1) // block * block


C1 = Workload("c1_gauss_2e20", 1 << 20, 1 << 20, 1 << 20, 4, 4, 30, 8, "f32", False, "gauss")
C2 = Workload("c2_resnet50", 25_557_032, 1 << 25, 1 << 25, 8, 4, 30, 8, "f32", True, "resnet50")
C3 = Workload("c3_vgg16", 138_357_544, 1 << 28, 1 << 20, 8, 4, 30, 8, "f32", False, "vgg16")
C4_B4 = Workload("c4_bert_large_b4", 336_000_000, _pad(336_000_000, 1 << 20), 1 << 20, 16, 4, 30, 16, "f32",
                 False, "bert")
C4_B2 = Workload("c4_bert_large_b2", 336_000_000, _pad(336_000_000, 1 << 20), 1 << 20, 16, 2, 8, 8, "f32",
                 False, "bert")
C5 = Workload("c5_gpt2_xl", 1_557_611_200, _pad(1_557_611_200, 1 << 22), 1 << 22, 32, 4, 30, 16, "bf16", True,
              "gpt2xl")

ALL = {w.name: w for w in (C1, C2, C3, C4_B4, C4_B2, C5)}

VGG16_FC_OFFSET = 14_714_688      # the convolutional parameters come first
VGG16_FC_SIZE = 102_760_448       # the largest fully connected layer


def shrink(w: Workload, blocks: int, n: Optional[int] = None) -> Workload:
    """The first `blocks` RHT blocks of a workload (same block size and distribution recipe), for parity
    runs that the CPU oracle can finish; optionally fewer workers."""
    d = min(w.d, blocks * w.block)
    return replace(w, name=f"{w.name}_first{blocks}", d=d, real=min(w.real, d), n=n if n is not None else w.n)


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _randn(n, gen, device):
    return torch.randn(n, generator=gen, device=device, dtype=torch.float32)


def _rand(n, gen, device):
    return torch.rand(n, generator=gen, device=device, dtype=torch.float32)


def resnet50_segments(real: int, seed: int = BASE_SEED) -> List[int]:
    """161 contiguous layer segments of seeded random sizes summing to `real`."""
    g = _gen("cpu", seed ^ 0x5E65)
    wts = -torch.log(torch.rand(161, generator=g, dtype=torch.float64))
    sizes = torch.floor(wts / wts.sum() * real).to(torch.int64)
    sizes = torch.clamp(sizes, min=1)
    sizes[-1] += real - int(sizes.sum())
    assert int(sizes.sum()) == real and int(sizes.min()) >= 1
    return [int(s) for s in sizes]


def gradient(w: Workload, worker: int, device="cpu", seed: int = BASE_SEED) -> torch.Tensor:
    """Worker `worker`'s padded gradient: float32 (or bfloat16) tensor of w.d values on `device`."""
    dev = torch.device(device)
    gen = _gen(dev, seed + worker)
    real = min(w.real, w.d)
    out = torch.zeros(w.d, dtype=torch.float32, device=dev)
    if w.kind == "gauss":
        out[:real] = _randn(real, gen, dev) * 1e-3
    elif w.kind == "vgg16":
        out[:real] = _randn(real, gen, dev) * 1e-3
        lo, hi = min(VGG16_FC_OFFSET, real), min(VGG16_FC_OFFSET + VGG16_FC_SIZE, real)
        out[lo:hi] *= 0.1                                  # N(0, (1e-4)^2) on the big FC layer
    elif w.kind == "resnet50":
        sizes = resnet50_segments(w.real, seed)
        gs = _gen("cpu", seed ^ 0xA11CE)
        scales = 10.0 ** (torch.rand(161, generator=gs, dtype=torch.float64) * 3.0 - 5.0)   # log-uniform [1e-5, 1e-2]
        pos = 0
        for sz, sc in zip(sizes, scales.tolist()):
            if pos >= real:
                break
            sz = min(sz, real - pos)
            u = _rand(sz, gen, dev) - 0.5                  # Laplace(0, s) by inverse CDF
            a = torch.clamp(2.0 * u.abs(), max=1.0 - 2.0 ** -24)   # a draw of exactly 0 would give log(0)
            out[pos:pos + sz] = -sc * torch.sign(u) * torch.log1p(-a)
            pos += sz
    elif w.kind == "bert":
        gs = _gen("cpu", seed ^ (0xBE27 + worker))
        sigma = float(10.0 ** (torch.rand(1, generator=gs, dtype=torch.float64) * 2.0 - 4.0))   # [1e-4, 1e-2]
        out[:real] = _randn(real, gen, dev) * sigma
        mask = _rand(real, gen, dev) < 1e-3                # 0.1 % outliers at 50 sigma
        sgn = torch.where(_rand(real, gen, dev) < 0.5, -1.0, 1.0)
        out[:real] = torch.where(mask, sgn * (50.0 * sigma), out[:real])
    elif w.kind == "gpt2xl":
        chunk = 1 << 26
        for pos in range(0, real, chunk):
            sz = min(chunk, real - pos)
            z = _randn(sz, gen, dev)
            chi = _randn(sz, gen, dev) ** 2 + _randn(sz, gen, dev) ** 2 + _randn(sz, gen, dev) ** 2
            out[pos:pos + sz] = z / torch.sqrt(chi / 3.0) * 1e-3      # Student-t, 3 degrees of freedom
    else:
        raise ValueError(w.kind)
    if w.dtype == "bf16":
        return out.to(torch.bfloat16)
    return out


def checksum(t: torch.Tensor) -> dict:
    """A few numbers that identify a generated buffer in logs."""
    f = t.to(torch.float64)
    return {"sum": float(f.sum()), "sumsq": float((f * f).sum()), "nonzero": int((t != 0).sum())}


def table_and_threshold(w: Workload):
    """(table, t_p) for a workload through the library's own host-side solver."""
    from . import api
    table, _ = api.thc_solve_table(w.b, w.g, w.p)
    return table, api.thc_threshold(w.p)


def bytes_per_coord(w: Workload) -> float:
    """Compulsory HBM bytes per (padded) coordinate for one full round: each datum crosses HBM once.
    compress: n * (input + [EF read + write] + packed);  aggregate: n * packed + sums;  decompress: sums + output."""
    in_b = 4 if w.dtype == "f32" else 2
    comp = w.n * (in_b + (8 if w.ef else 0) + w.b / 8)
    agg = w.n * w.b / 8 + w.agg_bits / 8
    dec = w.agg_bits / 8 + 4
    return comp + agg + dec


def moved_bytes_per_coord(w: Workload) -> float:
    """HBM bytes per (padded) coordinate the kernels actually move in one full round: every pass of a transform
    reads and writes the vector once (rocprofv3's FETCH_SIZE / WRITE_SIZE read exactly this on the VGG16-shaped
    workload).  A transform of 2^L coordinates takes the first pass (13 bits), the last pass (up to 9 bits) and,
    above L = 22, ceil((L - 13) / 7) - 1 passes in between."""
    in_b = 4 if w.dtype == "f32" else 2
    L = w.block.bit_length() - 1
    mids = 0 if L - 13 <= 9 else -(-(L - 13) // 7) - 1
    fwd = (in_b + (4 if w.ef else 0) + 4) + 8 * mids + (4 + w.b / 8)
    ef = (w.b / 8 + 4) + 8 * mids + (4 + in_b + 4 + 4) if w.ef else 0
    agg = w.n * w.b / 8 + w.agg_bits / 8
    dec = (w.agg_bits / 8 + 4) + 8 * mids + (4 + 4)
    return w.n * (fwd + ef) + agg + dec
