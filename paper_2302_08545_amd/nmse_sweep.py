"""NMSE of THC against the granularity g (the paper's App. C.4 experiment) on the GPU library.

A gradient is drawn from a lognormal distribution and given to every one of n workers; one THC round
(range, n x compress, aggregate, decompress) estimates the mean, which equals that gradient; the NMSE
||x - xhat||^2 / ||x||^2 (Sec. 2.1) is averaged over repeats.  The paper uses 10 workers, p = 1/1024 and
bit budgets 2, 3 and 4 and shows the curves only as a figure; this module prints the numbers, next to the
prediction for Gaussian rotated coordinates: table cost / n + truncation term.

    python -m paper_2302_08545_amd.nmse_sweep [--repeats 100] [--workers 10] [--log2d 20] [--p 0.0009765625]
"""
from __future__ import annotations

import argparse
import json
import math

from . import api


def truncation_term(t_p: float) -> float:
    """E[(|A| - t_p)^2 ; |A| > t_p] for A ~ N(0,1): what clamping to [-t_p, t_p] costs, in sigma^2 units."""
    phi = math.exp(-0.5 * t_p * t_p) / math.sqrt(2.0 * math.pi)
    tail = 0.5 * math.erfc(t_p / math.sqrt(2.0))
    return 2.0 * ((1.0 + t_p * t_p) * tail - t_p * phi)


def sweep(bs=(2, 3, 4), g_max=51, n=10, p=1.0 / 1024, log2d=20, repeats=100, device="cuda:0", seed=20230208):
    import torch
    d = 1 << log2d
    t_p = api.thc_threshold(p)
    trunc = truncation_term(t_p)
    gen = torch.Generator(device=device)
    rows = []
    ws = None
    out = torch.empty(d, dtype=torch.float32, device=device)
    range_M = torch.empty(1, dtype=torch.float32, device=device)
    for b in bs:
        for g in range(2 ** b - 1, g_max + 1):
            table, cost = api.thc_solve_table(b, g, p)
            agg_bits = max(1, math.ceil(math.log2(g * n + 1)))
            P = api.make_params(d, d, n, b, g, t_p, seed, table, agg_bits)
            need = api.thc_workspace_bytes(P)
            if ws is None or ws.numel() < need:
                ws = torch.empty(need, dtype=torch.uint8, device=device)
            packed = [torch.empty(d * b // 8, dtype=torch.uint8, device=device) for _ in range(n)]
            agg = torch.empty(d * agg_bits // 8, dtype=torch.uint8, device=device)
            gen.manual_seed(seed + 1000 * b + g)
            acc = 0.0
            for r in range(repeats):
                x = torch.randn(d, generator=gen, device=device, dtype=torch.float32).exp_()   # LogNormal(0, 1)
                grads = [x] * n                                   # the same gradient on every worker
                api.thc_compress_all(P, r, grads, None, range_M, packed, ws)
                api.thc_aggregate(P, packed, agg)
                api.thc_decompress(P, r, agg, range_M, out, ws)
                xd = x.double()
                acc += float(((xd - out.double()) ** 2).sum() / (xd * xd).sum())
            rows.append({"b": b, "g": g, "table": table, "nmse": acc / repeats,
                         "predicted": cost / n + trunc, "table_cost": cost})
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--repeats", type=int, default=100)
    ap.add_argument("--workers", type=int, default=10)
    ap.add_argument("--log2d", type=int, default=20)
    ap.add_argument("--p", type=float, default=1.0 / 1024)
    ap.add_argument("--gmax", type=int, default=51)
    ap.add_argument("--json", action="store_true")
    a = ap.parse_args()
    rows = sweep(n=a.workers, p=a.p, log2d=a.log2d, repeats=a.repeats, g_max=a.gmax)
    if a.json:
        print(json.dumps(rows))
        return
    print(f"# NMSE vs granularity: {a.workers} workers, p = {a.p:g}, d = 2^{a.log2d}, {a.repeats} repeats, lognormal gradient")
    print("| b | g | NMSE (measured) | predicted | table |")
    print("|---|---|---|---|---|")
    for r in rows:
        print(f"| {r['b']} | {r['g']} | {r['nmse']:.5f} | {r['predicted']:.5f} | {' '.join(map(str, r['table']))} |")


if __name__ == "__main__":
    main()
