"""Benchmark of the THC hot path on one MI355X.

A step is one full round (Alg. 3) for n workers whose buffers are resident in HBM: thc_compress_all (range + the n
workers' compressed streams), thc_aggregate, thc_decompress, with the round counter advancing.  The default workload
is the VGG16-shaped one (138,357,544 coordinates zero-padded to 2^28, 8 workers, b = 4, g = 30, RHT block 2^20).
Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X HBM3E
CPU_SHARE = 16             # host cores that go with one GPU of the box


def measured_traffic(workload_name):
    """Bytes the forward sweep moves between the L2s and memory per launch, from the tracked rocprofv3 counter
    summary (profiles/all_kernels_<workload>.txt, line `traffic_bytes_per_launch: N`), or None."""
    path = os.path.join(ROOT, "profiles", f"all_kernels_{workload_name}.txt")
    try:
        m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def profiled_kernel(workload_name, prefix):
    """(kernel name, launches per round, average microseconds per launch) of the first kernel whose name starts with
    `prefix` in the tracked rocprofv3 summary of the workload, or None."""
    path = os.path.join(ROOT, "profiles", f"all_kernels_{workload_name}.txt")
    try:
        text = open(path).read()
    except OSError:
        return None
    rounds = re.search(r"time over (\d+) rounds", text)
    m = re.search(r"^(" + re.escape(prefix) + r".*?\))\s+(\d+)\s+([0-9.]+)\s+([0-9.]+)", text, re.M)
    if not m or not rounds:
        return None
    return m.group(1), int(m.group(2)) / int(rounds.group(1)), float(m.group(4))


# ---------------------------------------------------------------------------------------------- oracle baseline
def _oracle_block_round(task):
    """One full round of the oracle on one block of all n workers (blocks are independent THC instances)."""
    import numpy as np
    from oracle import thc_oracle as o
    Pd, k, rnd, grads, efs = task
    P = o.Params(**Pd)
    j0 = k * P.block
    M = o.prepare_range(P, grads, efs)
    packed = [o.compress(P, i, rnd, grads[i], None if efs is None else efs[i], M, j0=j0)[0] for i in range(P.n)]
    Y = o.aggregate(P, packed)
    out = o.decompress(P, rnd, Y, M, j0=j0)
    return float(np.abs(out).sum())


def cpu_baseline(w, order, blocks_single=4, blocks_per_core=2, budget_coords=1 << 28):
    """The oracle as it stands, timed on the host before anything touches the GPU: the first blocks of the same
    workload, all n workers, one full round per block.  One process first, then a pool of the machine's host cores over
    independent blocks.  A bounded sample; whole-workload figures follow by linear extrapolation."""
    import multiprocessing as mp
    import numpy as np
    import torch
    from oracle import thc_oracle as o
    from paper_2302_08545_amd import workloads as wl
    cores = max(1, min(CPU_SHARE, os.cpu_count() or 1))
    per_block = w.block * w.n
    nblk = max(1, min(w.K, max(blocks_single, blocks_per_core * cores), budget_coords // per_block))
    ws = wl.shrink(w, nblk)
    grads = [wl.gradient(ws, i, device="cpu").to(dtype=torch.float32).numpy() for i in range(ws.n)]
    B = ws.block
    Pd = dict(d=B, block=B, n=ws.n, b=ws.b, g=ws.g, t_p=o.t_p_of(ws.p), seed=wl.RHT_SEED,
              table=o.solve_table(ws.b, ws.g, ws.p), agg_bits=ws.agg_bits, order=order)

    def task(k):
        sl = slice(k * B, (k + 1) * B)
        efs = [np.zeros(B, dtype=np.float32) for _ in range(ws.n)] if ws.ef else None
        return (Pd, k, 0, [g[sl] for g in grads], efs)

    n1 = min(blocks_single, nblk)
    t0 = time.perf_counter()
    for k in range(n1):
        _oracle_block_round(task(k))
    t1 = time.perf_counter() - t0
    t0 = time.perf_counter()
    with mp.get_context("fork").Pool(min(cores, nblk)) as pool:
        pool.map(_oracle_block_round, [task(k) for k in range(nblk)], chunksize=1)
    tp = time.perf_counter() - t0
    return {"value": nblk * B / tp, "unit": "coords/s", "cores": min(cores, nblk), "kind": "oracle",
            "host_cpu_count": os.cpu_count(),
            "one_thread_value": n1 * B / t1,
            "sample": f"first {nblk} block(s) of {B} coordinates x {ws.n} workers, one full round per block, in a pool of "
                      f"{min(cores, nblk)} processes: {tp:.2f} s; one process over {n1} block(s): {t1:.2f} s; whole-workload "
                      f"figures are linear extrapolations (blocks are independent)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3_vgg16")
    ap.add_argument("--blocks", type=int, default=0, help="use only the first N RHT blocks")
    ap.add_argument("--workers", type=int, default=0, help="override the number of workers (memory)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-order", choices=("ascending", "split"), default="split",
                    help="order of the butterfly stages (thc_params.stage_order)")
    ap.add_argument("--variant", choices=("thc", "uniform", "uniform-rotated"), default="thc",
                    help="thc: Alg. 3 (the headline).  uniform / uniform-rotated: Alg. 1 on the same workload "
                         "(identity table, g = 2^b - 1, min/max ranges), without / with the rotation")
    ap.add_argument("--graph", action="store_true",
                    help="capture one round in a HIP graph and replay it (the round counter then stays fixed): for "
                         "small vectors, where the launches of a round dominate")
    ap.add_argument("--block-log2", type=int, default=0, help="override the RHT block size (2^10 .. 2^27)")
    ap.add_argument("--agg-bits", type=int, default=0, help="override the width of the aggregated sums (1..16)")
    ap.add_argument("--calls", choices=("all", "each"), default="all",
                    help="all: thc_compress_all (range and the n workers' streams in one sweep, the headline).  "
                         "each: thc_prepare_range, then thc_compress once per worker")
    ap.add_argument("--group-log2", type=int, default=0,
                    help="thc_params.group_log2 (0 = the library's default; a value switches the single-launch sweep off)")
    ap.add_argument("--single-launch", action="store_true",
                    help="thc_params.single_launch: all passes of all blocks in one kernel launch, small workspace")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 1 GiB device-to-device copy five times and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (all n simulated workers live on it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    from paper_2302_08545_amd import workloads as wl
    w = wl.ALL[args.workload]
    if args.blocks:
        w = wl.shrink(w, args.blocks)
    if args.workers:
        w = wl.replace(w, n=args.workers, name=f"{w.name}_n{args.workers}")
    uniform = args.variant != "thc"
    rotate = args.variant == "uniform-rotated"
    if args.agg_bits:
        w = wl.replace(w, agg_bits=args.agg_bits)
    if args.block_log2:
        blk = 1 << args.block_log2
        w = wl.replace(w, block=blk, d=-(-w.d // blk) * blk)
    order_id = 1 if args.stage_order == "split" else 0

    # the oracle first: its process pool must exist before this process touches the GPU
    baseline = None
    if not uniform and not args.no_cpu_baseline and not args.calibrate_copy:
        baseline = cpu_baseline(w, order_id)

    import torch
    from paper_2302_08545_amd import api

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
    table, t_p = wl.table_and_threshold(w)
    if uniform:
        w = wl.replace(w, g=2 ** w.b - 1)
        table = list(range(2 ** w.b))
    seed = wl.RHT_SEED
    order = api.THC_ORDER_SPLIT if args.stage_order == "split" else api.THC_ORDER_ASCENDING
    L = api.make_params(w.d, w.block, w.n, w.b, w.g, t_p, seed, table, w.agg_bits,
                        api.THC_DTYPE_BF16 if w.dtype == "bf16" else api.THC_DTYPE_F32, order, 0, args.group_log2, int(args.single_launch))

    grads = [wl.gradient(w, i, device=dev) for i in range(w.n)]
    print("bench input checksums:", json.dumps({f"worker{i}": wl.checksum(grads[i][:1 << 24]) for i in (0, w.n - 1)}),
          file=sys.stderr, flush=True)
    efs = [torch.zeros(w.d, dtype=torch.float32, device=dev) for _ in range(w.n)] if w.ef else None
    ws_bytes = (api.thc_uniform_workspace_bytes(L, rotate) if uniform else api.thc_workspace_bytes(L, w.ef))
    ws = torch.zeros(ws_bytes, dtype=torch.uint8, device=dev)
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
    status = int(ws[:4].view(torch.int32).cpu()[0])
    assert uniform or status == 0, f"the single-launch sweep reported status {status}"

    per_step = dt / args.steps
    stage_ms = {name: sum(ev[k].elapsed_time(ev[k + 1]) for ev in events) / len(events)
                for k, name in enumerate(stage_names)}
    rounds_ms = sorted(ev[0].elapsed_time(ev[4]) for ev in events)   # each round by its own events
    bpc = wl.bytes_per_coord(w)
    in_bytes = 4 if w.dtype == "f32" else 2
    # Dominant launch: the forward sweep, thc_compress_all (one kernel launch that takes all workers' blocks through
    # first pass, range, last pass + quantizer [+ the error-feedback inverse]; a small launch before it clears its
    # counters).  Algorithmic bytes: every gradient (and error-feedback buffer) read once, the error-feedback buffer
    # written once, the packed indices written once.  Duration: HIP events around the call, on the launch stream.
    fwd_alg_bytes = w.n * w.d * (in_bytes + (8 if w.ef else 0) + w.b / 8)
    fwd_ms = stage_ms["prepare_range"] + stage_ms["compress"]
    achieved = fwd_alg_bytes / (fwd_ms * 1e-3) / 1e9
    default_config = (args.stage_order == "split" and not args.block_log2 and not args.agg_bits and args.calls == "all"
                      and not args.group_log2 and not args.blocks and not args.workers and not args.graph
                      and not args.single_launch)
    result = {
        "metric": "gradient coords/s (compress+aggregate+decompress), coordinates of the zero-padded vector",
        "value": w.d / per_step,
        "unit": "coords/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": per_step * 1e3,
        "ms_per_step_median": rounds_ms[len(rounds_ms) // 2],
        "ms_per_step_min": rounds_ms[0],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "d_padded": w.d, "d_real": w.real, "rht_block": w.block, "workers": w.n,
                   "b": w.b, "g": w.g, "agg_bits": w.agg_bits, "error_feedback": w.ef, "input": w.dtype,
                   "stage_order": args.stage_order, "variant": args.variant, "hip_graph": args.graph,
                   "calls": args.calls, "group_log2": args.group_log2, "single_launch": args.single_launch,
                   "workspace_bytes": ws_bytes},
        "value_real": w.real / per_step,        # the same time over the coordinates that carry data (no padding)
        "worker_coords_per_s": w.n * w.d / per_step,
        "effective_hbm_GBps": bpc * w.d / per_step / 1e9,
        "effective_hbm_frac": bpc * w.d / per_step / 1e9 / HBM_PEAK_GBPS,
        "compulsory_bytes_per_coord": bpc,
        # what two-pass transforms move between the L2s and memory or its cache, over the same time
        "moved_bytes_per_coord": wl.moved_bytes_per_coord(w),
        "moved_GBps": wl.moved_bytes_per_coord(w) * w.d / per_step / 1e9,
        "stage_ms": stage_ms,
        "roofline": {"bound": "hbm", "kernel": ("k_pipe_forward (thc_compress_all, single launch)" if args.single_launch else
                                "thc_compress_all: k_fwd_lo + k_range" + (" + k_mid" if w.block > 1 << 22 else "")
                                + " + k_fwd_hi_quant" + (" + k_inv_lo" + (" + k_mid" if w.block > 1 << 22 else "")
                                                         + " + k_inv_hi (error feedback)" if w.ef else "")
                                + " per group of blocks")
                     if args.calls == "all" else "thc_prepare_range + n x thc_compress", "achieved": achieved,
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS,
                     "algorithmic_bytes": fwd_alg_bytes, "launch_ms": fwd_ms,
                     "traffic": measured_traffic(w.name) if default_config else None},
    }
    pk = profiled_kernel(w.name, "k_fwd_lo") if default_config else None
    if pk is not None:
        # The sweep's largest kernel by itself, from the tracked rocprofv3 summary (not measured in this run): the
        # gradients (and error-feedback buffers) its launch reads, over its average duration.
        name, per_round, avg_us = pk
        lo_bytes = w.n * w.d * (in_bytes + (4 if w.ef else 0)) / per_round
        result["roofline"]["largest_kernel"] = {"name": name, "launches_per_round": per_round, "avg_us": avg_us,
                                                "algorithmic_bytes": lo_bytes,
                                                "frac": lo_bytes / (avg_us * 1e-6) / 1e9 / HBM_PEAK_GBPS,
                                                "source": f"profiles/all_kernels_{w.name}.txt"}
    if w.name == "c3_vgg16" and default_config:
        # Vector-ALU view of the same sweep: wave64 instructions it issues (rocprofv3 SQ_INSTS_VALU,
        # profiles/sq_counters_c3_vgg16.txt) against what 1024 SIMDs issue at one instruction per 4 cycles, 2.35 GHz
        insts = 4 * (242089984 + 231800832)
        result["alu_roofline"] = {"bound": "alu", "kernel": result["roofline"]["kernel"], "unit": "wave64 instructions/s",
                                  "achieved": insts / (fwd_ms * 1e-3), "peak": 1024 * 2.35e9 / 4,
                                  "frac": insts / (fwd_ms * 1e-3) / (1024 * 2.35e9 / 4)}
    if uniform:
        # Alg. 1 runs other kernels: the figures above that describe Alg. 3's passes do not apply
        for key in ("roofline", "moved_bytes_per_coord", "moved_GBps"):
            result[key] = None
    elif baseline is not None:
        result["cpu_baseline"] = baseline
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
