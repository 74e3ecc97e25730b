"""Lookup-table tool (Sec. 5.2, App. B): optimal tables T_{b,g,p} for every combination the paper mentions.

    python -m paper_2302_08545_amd.tables                # b = 1..4, g = 2^b-1..51, p in {1/32 ... 1/1024}
    python -m paper_2302_08545_amd.tables --check 3 12   # also run the exhaustive search of Alg. 4 for (b, g)
"""
from __future__ import annotations

import argparse
import time

from . import api

P_VALUES = (1 / 32, 1 / 64, 1 / 128, 1 / 256, 1 / 512, 1 / 1024)


def solve_all(bs=(1, 2, 3, 4), g_max=51, ps=P_VALUES):
    out = {}
    for b in bs:
        for g in range(2 ** b - 1, g_max + 1):
            for p in ps:
                out[(b, g, p)] = api.thc_solve_table(b, g, p)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gmax", type=int, default=51)
    ap.add_argument("--check", nargs=2, type=int, metavar=("B", "G"))
    a = ap.parse_args()
    if a.check:
        b, g = a.check
        for p in P_VALUES:
            t0 = time.perf_counter()
            tb, cb, cnt = api.thc_solve_table_bruteforce(b, g, p)
            t1 = time.perf_counter()
            td, cd = api.thc_solve_table(b, g, p)
            print(f"b={b} g={g} p=1/{round(1 / p)}: {cnt} candidates in {t1 - t0:.2f} s; exhaustive {tb} ({cb:.9f}); "
                  f"shortest path {td} ({cd:.9f}); {'equal' if tb == td else 'DIFFERENT'}")
        return
    t0 = time.perf_counter()
    tables = solve_all(g_max=a.gmax)
    dt = time.perf_counter() - t0
    print(f"# {len(tables)} tables in {dt:.2f} s")
    print("| b | g | p | cost (sigma^2) | table |")
    print("|---|---|---|---|---|")
    for (b, g, p), (t, c) in tables.items():
        print(f"| {b} | {g} | 1/{round(1 / p)} | {c:.6f} | {' '.join(map(str, t))} |")


if __name__ == "__main__":
    main()
