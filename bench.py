"""Benchmark of the THC hot path on one MI355X.

A step is one full round (Alg. 3) for n workers whose buffers are resident in HBM:
thc_prepare_range (x n fused), n x thc_compress, thc_aggregate, thc_decompress, with the round counter
advancing.  The default workload is the VGG16-shaped one (138,357,544 coordinates padded to 2^28, 8 workers,
b = 4, g = 30, RHT block 2^20).  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E

# HBM bytes per launch of the dominant kernel (k_fwd_lo) on the default workload, from two rocprofv3 --pmc
# runs of this file (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each scaled by what the same counter
# reads for the plain 1 GiB copy of --calibrate-copy (FETCH_SIZE x 2.0, WRITE_SIZE x 1.0).
# Summary and commands: profiles/k_fwd_lo_c3_vgg16_hbm_bytes.txt
MEASURED_TRAFFIC_BYTES = {"c3_vgg16": (4194371.2 * 2.0 + 8397262.9 * 1.0) * 1024.0}


def cpu_baseline(w, table, t_p, seed, order=0, budget_blocks=16):
    """The oracle as it stands, timed on the host on a bounded sample: the first block(s) of the same
    workload, all n workers, one full round."""
    import numpy as np
    from oracle import thc_oracle as o
    from paper_2302_08545_amd import workloads as wl
    ws = wl.shrink(w, budget_blocks)
    grads = [wl.gradient(ws, i, device="cpu").to(dtype=__import__("torch").float32).numpy() for i in range(ws.n)]
    efs = [np.zeros(ws.d, dtype=np.float32) for _ in range(ws.n)] if ws.ef else None
    P = o.Params(d=ws.d, block=ws.block, n=ws.n, b=ws.b, g=ws.g, t_p=t_p, seed=seed, table=table, agg_bits=ws.agg_bits,
                 order=order)
    t0 = time.perf_counter()
    o.thc_round(P, 0, grads, efs)
    dt = time.perf_counter() - t0
    return {"value": ws.d / dt, "unit": "coords/s", "cores": 1, "kind": "oracle",
            "sample": f"first {budget_blocks} block(s) of {ws.block} coordinates x {ws.n} workers, one full round, "
                      f"{dt:.2f} s of numpy on one host thread"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_vgg16")
    ap.add_argument("--blocks", type=int, default=0, help="use only the first N RHT blocks (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-order", choices=("ascending", "split"), default="split",
                    help="order of the butterfly stages (thc_params.stage_order)")
    ap.add_argument("--variant", choices=("thc", "uniform", "uniform-rotated"), default="thc",
                    help="thc: Alg. 3 (the headline).  uniform / uniform-rotated: Alg. 1 on the same workload "
                         "(identity table, g = 2^b - 1, min/max ranges), without / with the rotation")
    ap.add_argument("--graph", action="store_true",
                    help="capture one round in a HIP graph and replay it (the round counter then stays fixed): for "
                         "small vectors, where the dozen launches of a round dominate")
    ap.add_argument("--block-log2", type=int, default=0, help="override the RHT block size (2^10 .. 2^27)")
    ap.add_argument("--agg-bits", type=int, default=0, help="override the width of the aggregated sums (1..16)")
    ap.add_argument("--calls", choices=("all", "each"), default="all",
                    help="all: thc_compress_all (range and the n workers' streams in one sweep, the headline).  "
                         "each: thc_prepare_range, then thc_compress once per worker")
    ap.add_argument("--group-log2", type=int, default=0, help="thc_params.group_log2 (0 = the library's default)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device-to-device copy five times and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all n simulated workers live on it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2302_08545_amd import api
    from paper_2302_08545_amd import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    api.lib()                                   # fail loudly if the HIP library is missing
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)                      # reads 2^30 bytes and writes 2^30 bytes per launch
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": 1 << 30, "calibrate_copy_bytes_written": 1 << 30}))
        return
    w = wl.ALL[args.workload]
    if args.blocks:
        w = wl.shrink(w, args.blocks)
    table, t_p = wl.table_and_threshold(w)
    uniform = args.variant != "thc"
    rotate = args.variant == "uniform-rotated"
    if uniform:
        w = wl.replace(w, g=2 ** w.b - 1)
        table = list(range(2 ** w.b))
    if args.agg_bits:
        w = wl.replace(w, agg_bits=args.agg_bits)
    if args.block_log2:
        blk = 1 << args.block_log2
        w = wl.replace(w, block=blk, d=-(-w.d // blk) * blk)
    seed = wl.RHT_SEED
    order = api.THC_ORDER_SPLIT if args.stage_order == "split" else api.THC_ORDER_ASCENDING
    L = api.make_params(w.d, w.block, w.n, w.b, w.g, t_p, seed, table, w.agg_bits,
                        api.THC_DTYPE_BF16 if w.dtype == "bf16" else api.THC_DTYPE_F32, order, 0, args.group_log2)

    grads = [wl.gradient(w, i, device=dev) for i in range(w.n)]
    efs = [torch.zeros(w.d, dtype=torch.float32, device=dev) for _ in range(w.n)] if w.ef else None
    ws_bytes = (api.thc_uniform_workspace_bytes(L, rotate) if uniform else api.thc_workspace_bytes(L, w.ef))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    range_M = torch.zeros(w.K, dtype=torch.float32, device=dev)
    range_m = torch.zeros(w.K, dtype=torch.float32, device=dev)
    packed = [torch.zeros(w.d * w.b // 8, dtype=torch.uint8, device=dev) for _ in range(w.n)]
    agg = torch.zeros(w.d * w.agg_bits // 8, dtype=torch.uint8, device=dev)
    out = torch.zeros(w.d, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    stage_names = ("prepare_range", "compress", "aggregate", "decompress")
    events = []

    def step(rnd, timed):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)] if timed else None
        if timed:
            ev[0].record()
        if uniform:
            api.thc_uniform_prepare_range(L, rnd, grads, efs, rotate, range_m, range_M, ws)
        elif args.calls == "each":
            api.thc_prepare_range(L, grads, efs, range_M, ws)
        if timed:
            ev[1].record()
        if uniform:
            for i in range(w.n):
                api.thc_uniform_compress(L, i, rnd, grads[i], None if efs is None else efs[i], rotate, range_m, range_M,
                                         packed[i], ws)
        elif args.calls == "each":
            for i in range(w.n):
                api.thc_compress(L, i, rnd, grads[i], None if efs is None else efs[i], range_M, packed[i], ws)
        else:
            api.thc_compress_all(L, rnd, grads, efs, range_M, packed, ws)
        if timed:
            ev[2].record()
        api.thc_aggregate(L, packed, agg)
        if timed:
            ev[3].record()
        if uniform:
            api.thc_uniform_decompress(L, rnd, agg, rotate, range_m, range_M, out, ws)
        else:
            api.thc_decompress(L, rnd, agg, range_M, out, ws)
        if timed:
            ev[4].record()
            events.append(ev)

    for r in range(args.warmup):
        step(r, False)
    torch.cuda.synchronize()
    if args.graph:
        cap = torch.cuda.Stream()
        cap.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(cap):
            step(args.warmup, False)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=cap):
                step(args.warmup, False)
        torch.cuda.current_stream().wait_stream(cap)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for r in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        step(args.warmup, True)                 # one eager round for the per-stage split
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for r in range(args.steps):
            step(args.warmup + r, True)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    stage_ms = {name: sum(ev[k].elapsed_time(ev[k + 1]) for ev in events) / len(events)
                for k, name in enumerate(stage_names)}
    bpc = wl.bytes_per_coord(w)
    in_bytes = 4 if w.dtype == "f32" else 2
    # Dominant part: the forward sweep (per group of blocks: first pass of all workers, range, last pass + quantizer
    # of all workers [+ the error-feedback inverse]).  Its algorithmic bytes: every gradient (and error-feedback
    # buffer) read once, the error-feedback buffer written once, the packed indices written once.
    lo_alg_bytes = w.n * w.d * (in_bytes + (8 if w.ef else 0) + w.b / 8)
    lo_ms = stage_ms["prepare_range"] + stage_ms["compress"]
    achieved = lo_alg_bytes / (lo_ms * 1e-3) / 1e9
    result = {
        "metric": "gradient coords/s (compress+aggregate+decompress)",
        "value": w.d / (dt / args.steps),
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "d_padded": w.d, "d_real": w.real, "rht_block": w.block, "workers": w.n,
                   "b": w.b, "g": w.g, "agg_bits": w.agg_bits, "error_feedback": w.ef, "input": w.dtype,
                   "stage_order": args.stage_order, "variant": args.variant, "hip_graph": args.graph},
        "worker_coords_per_s": w.n * w.d / (dt / args.steps),
        "effective_hbm_GBps": bpc * w.d / (dt / args.steps) / 1e9,
        "effective_hbm_frac": bpc * w.d / (dt / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "compulsory_bytes_per_coord": bpc,
        # what the two-pass transforms really move (equal to the rocprofv3 counters on c3_vgg16), over the same time
        "moved_bytes_per_coord": wl.moved_bytes_per_coord(w),
        "moved_hbm_GBps": wl.moved_bytes_per_coord(w) * w.d / (dt / args.steps) / 1e9,
        "moved_hbm_frac": wl.moved_bytes_per_coord(w) * w.d / (dt / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "stage_ms": stage_ms,
        "roofline": {"bound": "hbm", "kernel": "forward sweep (k_fwd_lo + k_range + k_fwd_hi_quant per group)", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "algorithmic_bytes": lo_alg_bytes, "traffic": MEASURED_TRAFFIC_BYTES.get(w.name)},
    }
    if uniform:
        # Alg. 1 runs other kernels: the figures above that describe Alg. 3's passes do not apply
        for key in ("roofline", "moved_bytes_per_coord", "moved_hbm_GBps", "moved_hbm_frac"):
            result[key] = None
    elif not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, table, t_p, seed, order)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
