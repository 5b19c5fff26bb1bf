#!/usr/bin/env python3
"""Benchmark of the rank-n tensor transpose hot path on one MI355X.

A step is one pass over one batch of synthetic input: every permutation of the workload
(default: the rank-4 fp64 96^4 tensor with all 23 non-identity permutations) is executed
once through the C ABI, from a device-resident input into a device-resident output.  The
metric is the paper's bandwidth formula, 2 * vol * E / t (Section 3.1), in GB/s
(GB = 1e9 bytes), over the whole step.

Prints ONE JSON line.  `roofline` prices the tile kernel (the kernel every staged
transpose runs through) against the 8 TB/s HBM peak using its per-launch durations taken
with HIP events inside the timed region; `cpu_baseline` is the CPU oracle timed on this
box's host cores on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM traffic per launch of the tile kernel on the default workload, from rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE runs scaled by what the same counters read for the library's
# plain copy of known size (see profiles/tile_kernel_c2_96x96x96x96_fp64.txt, and
# profiles/tile_kernel_c7_square_sweep_fp32.txt for the square sweep: rows that start anywhere in
# a line fetch the partial lines at both ends of every row segment).  None = not measured.
TRAFFIC_BYTES_PER_LAUNCH = {"c2": 1358868800, "c7": 1921306400}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2,
                    help="workload family 1..5 (default 2); 6 = the paper's printed rank-8/rank-12 "
                         "shapes (Section 3.2), 7 = its square fp32 matrices of side 13952..13968")
    ap.add_argument("--accumulate", action="store_true",
                    help="time out = out + transpose(in) (Section 3.3); bytes = 3 * vol * E")
    ap.add_argument("--set2-perms", type=int, default=30, help="random permutations per shape for --config 6")
    ap.add_argument("--stride", type=int, default=1, help="take every n-th case of the family")
    ap.add_argument("--plan", choices=["heuristic", "measured"], default="heuristic")
    ap.add_argument("--max-candidates", type=int, default=48,
                    help="--plan measured: time this many of the best-scored candidates per case")
    ap.add_argument("--also-measured", action="store_true",
                    help="after the main pass, time the same step with measurement-selected plans")
    ap.add_argument("--also-graph", action="store_true",
                    help="additionally replay one step captured in a HIP graph (reported as graph_value)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--cases-out", default="", help="write per-case results (JSON lines) here")
    return ap.parse_args()


def cpu_baseline(cases, budget_s=12.0):
    """Time the CPU oracle (all host threads it uses) on a bounded sample of the cases."""
    import numpy as np

    import oracle
    from paper_1705_01598_amd import workloads as wl

    sample = cases[:: max(1, len(cases) // 8)][:8]
    total_bytes, total_t, names = 0, 0.0, []
    t_begin = time.perf_counter()
    for case in sample:
        a = wl.uniform_values(case)
        best = None
        for _ in range(2):
            t0 = time.perf_counter()
            oracle.transpose(a, case.dims, case.perm)
            dt = time.perf_counter() - t0
            best = dt if best is None or dt < best else best
            if time.perf_counter() - t_begin > budget_s:
                break
        total_bytes += case.bytes_moved
        total_t += best
        names.append(case.name)
        if time.perf_counter() - t_begin > budget_s:
            break
    return {"value": round(total_bytes / total_t / 1e9, 3), "unit": "GB/s",
            "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"{len(names)} of {len(cases)} cases ({', '.join(names)}), best of 2 each, "
                      f"2*vol*E/t summed over the sample"}


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1705_01598_amd import binding as B
    from paper_1705_01598_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()  # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.config == 6:
        cases = wl.set2(args.set2_perms)[:: args.stride]
    elif args.config == 7:
        cases = wl.square_sweep()[:: args.stride]
    else:
        cases = wl.all_configs()[args.config][:: args.stride]
    mem_ops = 3 if args.accumulate else 2
    run = B.tperm_execute_accumulate if args.accumulate else B.tperm_execute
    elem = cases[0].elem_size
    max_vol = max(c.volume for c in cases)
    stream = torch.cuda.current_stream().cuda_stream

    # device-resident input (uniform values of the first case's seed) and output; small
    # tensors rotate through several buffer pairs so that no launch finds its data in the
    # 256 MB last-level cache
    n_pairs = max(1, min(16, int((1 << 30) // (2 * max_vol * elem))))
    host = wl.uniform_values(wl.make_case(args.config, 0, (max_vol,), (0,), elem))
    bits = host.view(np.int64 if elem == 8 else np.int32)
    pairs = []
    for _ in range(n_pairs):
        a = torch.from_numpy(bits).to(dev)
        b = torch.empty_like(a)
        pairs.append((a, b))
    del host

    # measurement-based selection of tensors that fit the last-level cache is timed with a
    # 512 MiB scratch swept between executions, as the data will arrive from HBM in the timed loop
    scratch = torch.empty(512 << 20, dtype=torch.uint8, device=dev) if n_pairs > 1 else None

    def measured_plan(c, max_candidates):
        a, b = pairs[0]
        if scratch is not None:
            return B.tperm_plan_create_measured_cold(c.dims, c.perm, c.elem_size, a.data_ptr(), b.data_ptr(),
                                                     stream, scratch.data_ptr(), scratch.numel(), max_candidates)
        return B.tperm_plan_create_measured(c.dims, c.perm, c.elem_size, a.data_ptr(), b.data_ptr(),
                                            stream, max_candidates)

    plans = []
    for c in cases:
        if args.plan == "measured":
            plans.append(measured_plan(c, args.max_candidates))
        else:
            plans.append(B.tperm_plan_create(c.dims, c.perm, c.elem_size))
    infos = [p.describe() for p in plans]

    def one_step(step_idx, events=None):
        for i, plan in enumerate(plans):
            a, b = pairs[(step_idx * len(plans) + i) % n_pairs]
            if events is not None:
                events[i].record()
            run(plan, a.data_ptr(), b.data_ptr(), stream)
        if events is not None:
            events[len(plans)].record()

    for w in range(args.warmup):
        one_step(w)
    torch.cuda.synchronize()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(plans) + 1)]
          for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.steps):
        one_step(s, ev[s])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # per-launch durations from the events recorded inside the timed region
    dur_ms = np.array([[ev[s][i].elapsed_time(ev[s][i + 1]) for i in range(len(plans))]
                       for s in range(args.steps)])
    case_ms = np.median(dur_ms, axis=0)
    case_bytes = np.array([c.bytes_moved // 2 * mem_ops for c in cases], dtype=np.float64)
    case_gbs = case_bytes / case_ms / 1e6
    step_bytes = int(case_bytes.sum())
    value = step_bytes * args.steps / elapsed / 1e9

    tile_mask = np.array([i.kernel_class in (B.KERNEL_ROWCOPY, B.KERNEL_TILED, B.KERNEL_PACKED)
                          for i in infos])
    tile_bytes = case_bytes[tile_mask]
    tile_ms = dur_ms[:, tile_mask]
    achieved = float(tile_bytes.mean() / tile_ms.mean() / 1e6) if tile_mask.any() else 0.0
    traffic = TRAFFIC_BYTES_PER_LAUNCH.get(f"c{args.config}")

    # plain-copy ceiling of this machine, same size, for context (the paper normalises by a
    # measured STREAM figure, Section 3)
    a, b = pairs[0]
    nbytes = cases[0].volume * elem
    for _ in range(3):
        B.tperm_copy_bytes(a.data_ptr(), b.data_ptr(), nbytes, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(10):
        a, b = pairs[i % n_pairs]
        B.tperm_copy_bytes(a.data_ptr(), b.data_ptr(), nbytes, stream)
    e1.record()
    e1.synchronize()
    copy_gbs = 2 * nbytes * 10 / e0.elapsed_time(e1) / 1e6

    by_rank = {}
    for c, g in zip(cases, case_gbs):
        by_rank.setdefault(c.rank, []).append(float(g))
    rank_median = {str(r): round(float(np.median(v)), 1) for r, v in sorted(by_rank.items())}

    if args.cases_out:
        with open(args.cases_out, "w") as fh:
            for c, g, ms, info in zip(cases, case_gbs, case_ms, infos):
                fh.write(json.dumps({"case": c.name, "dims": c.dims, "perm": c.perm,
                                     "GBs": float(g), "us": float(ms) * 1e3,
                                     **B.info_dict(info)}) + "\n")

    workload_names = {1: "rank-2 fp64 2048x2048 transpose", 2: "rank-4 fp64 96^4, all 23 non-identity permutations",
                      3: "rank-6 fp64 ~2^26 elements, 20 seeded cases", 4: "rank sweep 2..12 fp64 ~2^26 elements, 330 seeded cases",
                      5: "fp32 contraction-feeding transposes 8^8 and 16^6, 80 seeded permutations",
                      6: "the paper's rank-8 (205M el) and rank-12 (328M el) fp64 shapes, seeded permutations + trivial + reverse",
                      7: "square fp32 matrices, side 13952..13968"}
    result = {
        "metric": "transpose GB/s (read+write bytes / time) and % of MI355X HBM peak, median/rank",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64" if elem == 8 else "f32",
        "data": "synthetic",
        "config": {"workload": workload_names[args.config], "cases": len(cases),
                   "bytes_per_step": step_bytes, "plan": args.plan, "buffer_pairs": n_pairs,
                   "mode": "accumulate (3 memory ops per element)" if args.accumulate else "transpose"},
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
        "case_median_GBs": round(float(np.median(case_gbs)), 1),
        "case_min_GBs": round(float(case_gbs.min()), 1),
        "case_max_GBs": round(float(case_gbs.max()), 1),
        "median_pct_hbm_peak": round(100.0 * float(np.median(case_gbs)) / HBM_PEAK_GBS, 2),
        "rank_median_GBs": rank_median,
        "copy_ceiling_GBs": round(copy_gbs, 1),
        "kernels": {B.KERNEL_NAMES[k]: int(sum(1 for i in infos if i.kernel_class == k))
                    for k in sorted({i.kernel_class for i in infos})},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "kernel": "tperm::tile_kernel",
                     "avg_launch_us": round(float(tile_ms.mean()) * 1e3, 2) if tile_mask.any() else None},
    }
    if args.also_measured and args.plan == "heuristic":
        # Section 2.3's other selection scheme, for comparison: plans chosen by timing every
        # candidate once at plan creation (outside any timed region)
        mplans = [measured_plan(c, 64) for c in cases]
        plans[:] = mplans
        for w in range(args.warmup):
            one_step(w)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            one_step(s)
        torch.cuda.synchronize()
        result["measured_plans_value"] = round(step_bytes * args.steps / (time.perf_counter() - t0) / 1e9, 1)
    if args.also_graph:
        # the same step as a HIP graph: what a caller with a fixed sequence of transposes gets
        # once the gaps between dependent launches are gone (one buffer pair per launch as in
        # the eager loop; the first use of every plan happened above, outside the capture)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            gs = torch.cuda.current_stream().cuda_stream
            for i, plan in enumerate(plans):
                a, b = pairs[i % n_pairs]
                run(plan, a.data_ptr(), b.data_ptr(), gs)
        for w in range(max(1, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["graph_value"] = round(step_bytes * args.steps / (time.perf_counter() - t0) / 1e9, 1)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cases)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
