#!/usr/bin/env python3
"""Benchmark of the rank-n tensor transpose hot path on one MI355X.

A step is one pass over one batch of synthetic input: every permutation of the workload
(headline: the rank-4 fp64 96^4 tensor with all 23 non-identity permutations) is executed
once through the C ABI, from a device-resident input into a device-resident output.  The
metric is the paper's bandwidth formula, 2 * vol * E / t (Section 3.1), in GB/s
(GB = 1e9 bytes), over the whole step.

Prints ONE JSON line.  `value` and the top-level fields describe the headline workload.
Without --config the other four workload families are timed as well, each with the same
harness, and reported under `per_config` (aggregate, per-case median / minimum, median per
rank and the ratio between the best and the worst rank median, event-timed fraction of the
HBM peak), and one case of every family is compared with the CPU oracle over the whole
tensor after the timed region (`bit_exact`).  `roofline` prices the tile kernel (the kernel
every staged transpose runs through) against the 8 TB/s HBM peak: algorithmic bytes per launch
over its average launch duration, which is the time between two HIP events that bracket the
timed region divided by the number of launches (per-case figures come from a second pass with
an event between every two launches, outside the timed region); `cpu_baseline` is the CPU oracle
timed on this machine's host cores on a bounded sample of the headline workload, with all the
threads it uses and with one.
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
HEADLINE = 2

# HBM traffic per launch of the tile kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# scaled by what the same counters read for the library's plain copy of known size.  These are
# figures copied from the named summaries, not something this run measures.
TRAFFIC = {
    2: (1359022760, "profiles/tile_kernel_c2_96x96x96x96_fp64.txt"),
    7: (1921306400, "profiles/tile_kernel_c7_square_sweep_fp32.txt"),
}

WORKLOAD_NAMES = {
    1: "rank-2 fp64 2048x2048 transpose",
    2: "rank-4 fp64 96^4, all 23 non-identity permutations",
    3: "rank-6 fp64 ~2^26 elements, 20 seeded cases",
    4: "rank sweep 2..12 fp64 ~2^26 elements, 330 seeded cases",
    5: "fp32 contraction-feeding transposes 8^8 and 16^6, 80 seeded permutations",
    6: "the paper's rank-8 (205M el) and rank-12 (328M el) fp64 shapes, seeded permutations + trivial + reverse",
    7: "square fp32 matrices, side 13952..13968",
    8: "held-out selector check: ranks 2..12, 2^25 and 2^27 elements, both element sizes, fresh seeds",
    9: "tensors of 4 GiB and more (4.0-8.0 GiB), both element sizes",
    10: "selector check on round extents: ranks 2-3, extents multiples of 2..16 elements, both element sizes",
}
# steps / warm-up of the families timed beside the headline one (their steps take 0.02-70 ms)
SIDE_STEPS = {1: (200, 20), 3: (10, 2), 4: (5, 1), 5: (20, 3)}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=0,
                    help="time one workload family only: 1..5; 6 = the paper's printed rank-8/rank-12 "
                         "shapes (Section 3.2), 7 = its square fp32 matrices of side 13952..13968, "
                         "8 = held-out shapes for the selector check, 9 = tensors of 4 GiB and more, "
                         "10 = round extents for the selector check.  Default: family 2 as the "
                         "headline, families 1, 3, 4, 5 beside it under per_config")
    ap.add_argument("--accumulate", action="store_true",
                    help="time out = out + transpose(in) (Section 3.3); bytes = 3 * vol * E")
    ap.add_argument("--set2-perms", type=int, default=30, help="random permutations per shape for --config 6")
    ap.add_argument("--stride", type=int, default=1, help="take every n-th case of the family")
    ap.add_argument("--plan", choices=["heuristic", "measured"], default="heuristic")
    ap.add_argument("--selector", choices=["fitted", "model"], default="fitted",
                    help="--plan heuristic: which host-side selector picks the tile: the fitted cost estimate "
                         "(default) or the analytical model of Section 2.3 re-derived for MI355X")
    ap.add_argument("--max-candidates", type=int, default=48,
                    help="--plan measured: time this many of the best-scored candidates per case")
    ap.add_argument("--also-measured", action="store_true",
                    help="after the main pass, time the same step with measurement-selected plans")
    ap.add_argument("--also-graph", action="store_true",
                    help="additionally replay one step captured in a HIP graph (reported as graph_value)")
    ap.add_argument("--also-two-streams", action="store_true",
                    help="additionally run the steps with the launches alternating between two streams and two "
                         "output buffers, so that one transpose starts while the other drains (reported as "
                         "two_stream_value; never the headline)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--no-verify", action="store_true", help="skip the whole-tensor oracle comparison")
    ap.add_argument("--cases-out", default="", help="write per-case results (JSON lines) here")
    ap.add_argument("--profile-pass", action="store_true",
                    help="for runs under rocprofv3: launch every case of the family once, in order, in two "
                         "passes (the second is the one to read), then the library's plain copy of the first "
                         "case's size three times (the known-size launch that counter readings are scaled "
                         "by), write the cases' plans to --cases-out and stop; no timing, no JSON line")
    return ap.parse_args()


def cpu_baseline(cases, budget_s=12.0):
    """Time the CPU oracle on a bounded sample of the cases: with all the host threads it
    uses, and (on the first two cases of the sample) with one thread."""
    import oracle
    from paper_1705_01598_amd import workloads as wl

    sample = cases[:: max(1, len(cases) // 8)][:8]
    total_bytes, total_t, names = 0, 0.0, []
    one_bytes, one_t, one_names = 0, 0.0, []
    t_begin = time.perf_counter()
    for n, case in enumerate(sample):
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
        if n < 2:
            t0 = time.perf_counter()
            oracle.transpose(a, case.dims, case.perm, nthreads=1)
            one_t += time.perf_counter() - t0
            one_bytes += case.bytes_moved
            one_names.append(case.name)
        if time.perf_counter() - t_begin > budget_s:
            break
    return {"value": round(total_bytes / total_t / 1e9, 3), "unit": "GB/s",
            "cores": oracle.max_threads(), "kind": "oracle",
            "sample": f"{len(names)} of {len(cases)} cases ({', '.join(names)}), best of 2 each, "
                      f"2*vol*E/t summed over the sample",
            "single_thread": {"value": round(one_bytes / one_t / 1e9, 3), "unit": "GB/s", "cores": 1,
                              "sample": f"{', '.join(one_names)}, one run each"}}


def family(args, config):
    from paper_1705_01598_amd import workloads as wl
    if config == 6:
        return wl.set2(args.set2_perms)[:: args.stride]
    if config == 7:
        return wl.square_sweep()[:: args.stride]
    if config == 8:
        return wl.heldout()[:: args.stride]
    if config == 9:
        return wl.large_tensors()[:: args.stride]
    if config == 10:
        return wl.even_extents()[:: args.stride]
    return wl.all_configs()[config][:: args.stride]


class Harness:
    """Device buffers, plans and the timed loop of one workload family."""

    def __init__(self, args, config, cases):
        import numpy as np
        import torch
        from paper_1705_01598_amd import binding as B
        from paper_1705_01598_amd import workloads as wl
        self.np, self.torch, self.B, self.wl = np, torch, B, wl
        self.args, self.config, self.cases = args, config, cases
        self.mem_ops = 3 if args.accumulate else 2
        self.run = B.tperm_execute_accumulate if args.accumulate else B.tperm_execute
        self.stream = torch.cuda.current_stream().cuda_stream
        dev = torch.device("cuda:0")
        # device-resident input (uniform values of the family's first seed) and output: one
        # buffer each, at least 512 MiB, so that a small tensor rotates through up to 16
        # places in them and no launch finds its data in the 256 MB last-level cache
        max_bytes = max(c.volume * c.elem_size for c in cases)
        buf_bytes = max(max_bytes, 512 << 20)
        fp32 = all(c.elem_size == 4 for c in cases)
        host = wl.uniform_values(wl.make_case(config, 0, (buf_bytes // (4 if fp32 else 8),), (0,), 4 if fp32 else 8))
        self.a = torch.from_numpy(host.view(np.int32 if fp32 else np.int64)).to(dev)
        self.b = torch.empty_like(self.a)
        del host
        # byte distance between the places of case i, and how many there are
        self.place = [(c.volume * c.elem_size + 4095) // 4096 * 4096 for c in cases]
        self.places = [max(1, min(16, buf_bytes // p)) for p in self.place]
        self.n_pairs = self.places[0]
        # measurement-based selection of tensors that fit the last-level cache is timed with a
        # 512 MiB scratch swept between executions, as the data will arrive from HBM in the timed loop
        self.scratch = torch.empty(512 << 20, dtype=torch.uint8, device=dev) \
            if (self.n_pairs > 1 and (args.plan == "measured" or args.also_measured)) else None
        def heuristic(c):
            if args.selector == "model":
                return B.tperm_plan_create_ex(c.dims, c.perm, c.elem_size, selector=1)
            return B.tperm_plan_create(c.dims, c.perm, c.elem_size)
        self.plans = [self.measured_plan(c, args.max_candidates) if args.plan == "measured" else heuristic(c)
                      for c in cases]
        self.infos = [p.describe() for p in self.plans]

    def measured_plan(self, c, max_candidates):
        B = self.B
        a, b = self.a, self.b
        if self.scratch is not None:
            return B.tperm_plan_create_measured_cold(c.dims, c.perm, c.elem_size, a.data_ptr(), b.data_ptr(),
                                                     self.stream, self.scratch.data_ptr(), self.scratch.numel(),
                                                     max_candidates)
        return B.tperm_plan_create_measured(c.dims, c.perm, c.elem_size, a.data_ptr(), b.data_ptr(),
                                            self.stream, max_candidates)

    def one_step(self, step_idx, events=None, stream=None):
        stream = self.stream if stream is None else stream
        pa, pb = self.a.data_ptr(), self.b.data_ptr()
        for i, plan in enumerate(self.plans):
            off = ((step_idx * len(self.plans) + i) % self.places[i]) * self.place[i]
            if events is not None:
                events[i].record()
            self.run(plan, pa + off, pb + off, stream)
        if events is not None:
            events[len(self.plans)].record()

    def timed(self, steps, warmup):
        """K steps between two synchronisations, with one HIP event in front of the first launch
        and one behind the last (on the stream the kernels run on).  Returns (wall seconds,
        event milliseconds over the K steps)."""
        torch = self.torch
        for w in range(warmup):
            self.one_step(w)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for s in range(steps):
            self.one_step(s)
        e1.record()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        return elapsed, e0.elapsed_time(e1)

    def per_case_ms(self, reps):
        """Per-case launch durations [reps x cases], in a pass of its own outside the timed
        region: every case is launched `batch` times back to back (rotating through its places
        in the buffers) between two events, and the batch time is divided by `batch`.  An event
        between every two launches would cost about 3 us per launch, which launches of 15-30 us
        feel; batches keep that below 1 %."""
        torch, np = self.torch, self.np
        pa, pb = self.a.data_ptr(), self.b.data_ptr()
        out = np.zeros((reps, len(self.plans)))
        for r in range(reps):
            evs = []
            for i, plan in enumerate(self.plans):
                batch = 4 if self.place[i] >= (256 << 20) else 16
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for k in range(batch):
                    off = ((r * batch + k) % self.places[i]) * self.place[i]
                    self.run(plan, pa + off, pb + off, self.stream)
                e1.record()
                evs.append((e0, e1, batch))
            torch.cuda.synchronize()
            out[r] = [e0.elapsed_time(e1) / batch for e0, e1, batch in evs]
        return out

    def copy_ceiling(self):
        """Plain-copy rate of this machine at the family's first size (the paper normalises by a
        measured STREAM figure, Section 3)."""
        torch, B = self.torch, self.B
        nbytes = self.cases[0].volume * self.cases[0].elem_size
        pa, pb = self.a.data_ptr(), self.b.data_ptr()
        for _ in range(3):
            B.tperm_copy_bytes(pa, pb, nbytes, self.stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(10):
            off = (i % self.places[0]) * self.place[0]
            B.tperm_copy_bytes(pa + off, pb + off, nbytes, self.stream)
        e1.record()
        e1.synchronize()
        return 2 * nbytes * 10 / e0.elapsed_time(e1) / 1e6

    def verify(self, index):
        """Whole-tensor, bit-for-bit comparison of one case with the CPU oracle (scrambled index
        stamps as input; outside every timed region)."""
        import oracle
        torch, np, wl = self.torch, self.np, self.wl
        case, plan = self.cases[index], self.plans[index]
        a = wl.scrambled_stamp_values(case.volume, case.elem_size)
        sign = np.int64 if case.elem_size == 8 else np.int32
        a_dev = torch.from_numpy(a.view(sign)).cuda()
        if self.args.accumulate:
            b = wl.uniform_values(case)
            out = torch.from_numpy(b.view(sign)).cuda()
            ref = oracle.transpose_accumulate(a.view(b.dtype), b, case.dims, case.perm)
        else:
            out = torch.full((case.volume,), -1, dtype=a_dev.dtype, device="cuda")
            ref = oracle.transpose(a, case.dims, case.perm)
        self.run(plan, a_dev.data_ptr(), out.data_ptr(), self.stream)
        torch.cuda.synchronize()
        ok = bool(torch.equal(out, torch.from_numpy(ref.view(sign)).cuda()))
        return {"case": case.name, "elements": case.volume, "bit_exact": ok}

    def summary(self, steps, warmup):
        """Time the family and condense the result."""
        np, B = self.np, self.B
        elapsed, region_ms = self.timed(steps, warmup)
        dur_ms = self.per_case_ms(3)
        cases, infos = self.cases, self.infos
        case_ms = np.median(dur_ms, axis=0)
        case_bytes = np.array([c.bytes_moved // 2 * self.mem_ops for c in cases], dtype=np.float64)
        case_gbs = case_bytes / case_ms / 1e6
        step_bytes = int(case_bytes.sum())
        value = step_bytes * steps / elapsed / 1e9
        tile_mask = np.array([i.kernel_class in (B.KERNEL_ROWCOPY, B.KERNEL_TILED, B.KERNEL_PACKED)
                              for i in infos])
        achieved, avg_us = 0.0, None
        if tile_mask.all():
            # every launch of the timed region is the tile kernel: its average duration is the
            # event time over the region divided by the number of launches
            avg_ms = region_ms / (steps * len(cases))
            achieved = float(case_bytes.mean() / avg_ms / 1e6)
            avg_us = round(avg_ms * 1e3, 2)
        elif tile_mask.any():
            # mixed with plain copies: take the tile kernel's share from the per-launch events
            achieved = float(case_bytes[tile_mask].mean() / dur_ms[:, tile_mask].mean() / 1e6)
            avg_us = round(float(dur_ms[:, tile_mask].mean()) * 1e3, 2)
        by_rank = {}
        for c, g in zip(cases, case_gbs):
            by_rank.setdefault(c.rank, []).append(float(g))
        rank_median = {str(r): round(float(np.median(v)), 1) for r, v in sorted(by_rank.items())}
        med = list(rank_median.values())
        out = {
            "workload": WORKLOAD_NAMES[self.config], "cases": len(cases), "steps": steps, "warmup": warmup,
            "dtype": "f64" if cases[0].elem_size == 8 else "f32",
            "value": round(value, 1), "ms_per_step": round(elapsed / steps * 1e3, 4),
            "bytes_per_step": step_bytes, "buffer_pairs": self.n_pairs,
            "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBS, 2),
            "case_median_GBs": round(float(np.median(case_gbs)), 1),
            "case_min_GBs": round(float(case_gbs.min()), 1),
            "case_max_GBs": round(float(case_gbs.max()), 1),
            "median_pct_hbm_peak": round(100.0 * float(np.median(case_gbs)) / HBM_PEAK_GBS, 2),
            "rank_median_GBs": rank_median,
            "rank_median_max_over_min": round(max(med) / min(med), 3),
            "tile_kernel_achieved_GBs": round(achieved, 1),
            "tile_kernel_frac": round(achieved / HBM_PEAK_GBS, 4),
            "tile_kernel_avg_launch_us": avg_us,
            "kernels": {B.KERNEL_NAMES[k]: int(sum(1 for i in infos if i.kernel_class == k))
                        for k in sorted({i.kernel_class for i in infos})},
        }
        lo, hi = str(min(by_rank)), str(max(by_rank))
        if lo != hi:
            out["lowest_vs_highest_rank"] = {"rank": [int(lo), int(hi)], "median_GBs": [rank_median[lo], rank_median[hi]],
                                             "ratio": round(max(rank_median[lo], rank_median[hi]) /
                                                            min(rank_median[lo], rank_median[hi]), 3)}
        self.case_gbs, self.case_ms = case_gbs, case_ms
        return out


def device_memory_figures(torch):
    """What the device itself reports about its memory system, next to the vendor's 8 TB/s."""
    from paper_1705_01598_amd import binding as B
    p = torch.cuda.get_device_properties(0)
    out = {"name": p.name, "l2_cache_bytes": getattr(p, "L2_cache_size", None)}
    out.update(B.tperm_device_memory_info())
    width, clock_khz = out["memory_bus_width_bits"], out["memory_clock_kHz"]
    if width and clock_khz:
        # double data rate: two transfers per reported clock
        out["bus_width_x_clock_x2_GBs"] = round(width / 8 * clock_khz * 1e3 * 2 / 1e9, 1)
    return out


def large_tensor_sample(torch, steps=12):
    """One tensor beyond 4 GiB (byte offsets no longer fit the 32-bit operands of buffer
    addressing; the plan reports large = 1): the 32768 x 32768 fp64 matrix transpose, 8 GiB each
    way, timed like every other case (two events around back-to-back launches)."""
    from paper_1705_01598_amd import binding as B
    dims, perm, elem = (1 << 15, 1 << 15), (1, 0), 8
    nbytes = dims[0] * dims[1] * elem
    a = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    b = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    a.random_(0, 255)
    plan = B.tperm_plan_create(dims, perm, elem)
    info = plan.describe()
    stream = torch.cuda.current_stream().cuda_stream
    for _ in range(4):
        B.tperm_execute(plan, a.data_ptr(), b.data_ptr(), stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(steps):
        B.tperm_execute(plan, a.data_ptr(), b.data_ptr(), stream)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    # checked on the device: a transpose moves every element once, none lost or duplicated
    verdict = torch.zeros(1, dtype=torch.int64, device="cuda:0")
    ws = torch.empty(B.verify_workspace_bytes(dims[0] * dims[1]), dtype=torch.uint8, device="cuda:0")
    B.tperm_execute_verified(plan, a.data_ptr(), b.data_ptr(), stream, verdict.data_ptr(), ws.data_ptr(), ws.numel())
    torch.cuda.synchronize()
    out = {"workload": "32768 x 32768 fp64 matrix transpose, 8 GiB each way", "large": int(info.large),
           "GBs": round(2.0 * nbytes / ms / 1e6, 1), "ms": round(ms, 3), "multiset_verdict": int(verdict.item())}
    del a, b, ws
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_1705_01598_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()  # fails loudly if the HIP library is missing
    torch.cuda.set_device(0)

    config = args.config or HEADLINE
    cases = family(args, config)
    h = Harness(args, config, cases)
    if args.profile_pass:
        for p in range(2):
            h.one_step(p)
            torch.cuda.synchronize()
        nbytes = cases[0].volume * cases[0].elem_size
        for _ in range(3):
            B.tperm_copy_bytes(h.a.data_ptr(), h.b.data_ptr(), nbytes, h.stream)
        torch.cuda.synchronize()
        if args.cases_out:
            with open(args.cases_out, "w") as fh:
                for c, info in zip(cases, h.infos):
                    fh.write(json.dumps({"case": c.name, "dims": c.dims, "perm": c.perm, "elem": c.elem_size,
                                         **B.info_dict(info)}) + "\n")
        return
    s = h.summary(args.steps, args.warmup)
    copy_gbs = h.copy_ceiling()
    traffic, traffic_source = TRAFFIC.get(config, (None, None))
    if args.plan != "heuristic" or args.accumulate or args.stride != 1:
        traffic, traffic_source = None, None

    if args.cases_out:
        with open(args.cases_out, "w") as fh:
            for c, g, ms, info in zip(cases, h.case_gbs, h.case_ms, h.infos):
                fh.write(json.dumps({"case": c.name, "dims": c.dims, "perm": c.perm, "elem": c.elem_size,
                                     "GBs": float(g), "us": float(ms) * 1e3,
                                     **B.info_dict(info)}) + "\n")

    result = {
        "metric": "transpose GB/s (read+write bytes / time) and % of MI355X HBM peak, median/rank",
        "value": s["value"],
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": s["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": s["dtype"],
        "data": "synthetic",
        "config": {"workload": s["workload"], "cases": len(cases),
                   "bytes_per_step": s["bytes_per_step"], "plan": args.plan if args.plan == "measured" or args.selector == "fitted" else "heuristic (analytical model)", "buffer_pairs": h.n_pairs,
                   "mode": "accumulate (3 memory ops per element)" if args.accumulate else "transpose"},
        "pct_hbm_peak": s["pct_hbm_peak"],
        "case_median_GBs": s["case_median_GBs"],
        "case_min_GBs": s["case_min_GBs"],
        "case_max_GBs": s["case_max_GBs"],
        "median_pct_hbm_peak": s["median_pct_hbm_peak"],
        "rank_median_GBs": s["rank_median_GBs"],
        "copy_ceiling_GBs": round(copy_gbs, 1),
        "kernels": s["kernels"],
        "device": device_memory_figures(torch),
        "roofline": {"bound": "hbm", "achieved": s["tile_kernel_achieved_GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": s["tile_kernel_frac"],
                     "traffic": traffic, "traffic_source": traffic_source, "kernel": "tperm::tile_kernel",
                     "avg_launch_us": s["tile_kernel_avg_launch_us"]},
    }
    if config in (8, 10) and args.plan == "heuristic":
        # selector check: the same cases with measurement-selected plans, case by case
        heur = h.case_gbs.copy()
        h.plans[:] = [h.measured_plan(c, 0) for c in cases]
        h.infos = [p.describe() for p in h.plans]
        h.summary(args.steps, args.warmup)
        ratio = heur / h.case_gbs
        import numpy as np
        result["heuristic_over_measured"] = {"mean": round(float(ratio.mean()), 4), "median": round(float(np.median(ratio)), 4),
                                             "min": round(float(ratio.min()), 4),
                                             "worst_case": cases[int(ratio.argmin())].name}
    if args.also_measured and args.plan == "heuristic":
        # Section 2.3's other selection scheme, for comparison: plans chosen by timing every
        # candidate once at plan creation (outside any timed region)
        if h.n_pairs > 1 and h.scratch is None:
            h.scratch = torch.empty(512 << 20, dtype=torch.uint8, device="cuda:0")
        h.plans[:] = [h.measured_plan(c, 64) for c in cases]
        elapsed, _ = h.timed(args.steps, args.warmup)
        result["measured_plans_value"] = round(s["bytes_per_step"] * args.steps / elapsed / 1e9, 1)
    if args.also_two_streams:
        # independent transposes on two streams, each stream with an output buffer of its own:
        # the first workgroups of one launch take the compute units the other's last ones leave
        b2 = torch.empty_like(h.b)
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        outs = [h.b.data_ptr(), b2.data_ptr()]

        def two_stream_step(k):
            for i, plan in enumerate(h.plans):
                off = ((k * len(h.plans) + i) % h.places[i]) * h.place[i]
                h.run(plan, h.a.data_ptr() + off, outs[i % 2] + off, streams[i % 2].cuda_stream)
        torch.cuda.synchronize()
        for w in range(max(1, args.warmup)):
            two_stream_step(w)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            two_stream_step(k)
        torch.cuda.synchronize()
        result["two_stream_value"] = round(s["bytes_per_step"] * args.steps / (time.perf_counter() - t0) / 1e9, 1)
        del b2
    if args.also_graph:
        # the same step as a HIP graph: what a caller with a fixed sequence of transposes gets
        # once the gaps between dependent launches are gone (one buffer pair per launch as in
        # the eager loop; the first use of every plan happened above, outside the capture)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            h.one_step(0, stream=torch.cuda.current_stream().cuda_stream)
        for w in range(max(1, args.warmup)):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        result["graph_value"] = round(s["bytes_per_step"] * args.steps / (time.perf_counter() - t0) / 1e9, 1)

    checks = []
    if not args.no_verify and args.plan == "heuristic":
        checks.append(h.verify(len(cases) // 2))
    if args.config == 0:
        # the other four families, same harness, each with its own buffers
        per = {f"c{HEADLINE}": {k: v for k, v in s.items()}}
        del h
        torch.cuda.empty_cache()
        for other, (steps, warmup) in SIDE_STEPS.items():
            oc = family(args, other)
            oh = Harness(args, other, oc)
            per[f"c{other}"] = oh.summary(steps, warmup)
            per[f"c{other}"]["copy_ceiling_GBs"] = round(oh.copy_ceiling(), 1)
            if not args.no_verify and args.plan == "heuristic":
                checks.append(oh.verify(len(oc) // 2))
            del oh
            torch.cuda.empty_cache()
        result["per_config"] = dict(sorted(per.items()))
        result["large_tensor"] = large_tensor_sample(torch)
        medians = [v["case_median_GBs"] for v in per.values()]
        result["all_configs_min_case_median_pct_hbm_peak"] = round(100.0 * min(medians) / HBM_PEAK_GBS, 2)
    if checks:
        result["verified"] = checks
        if not all(c["bit_exact"] for c in checks):
            print("bench.py: a timed plan does not reproduce the CPU oracle: " + json.dumps(checks), file=sys.stderr)
            sys.exit(1)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cases)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
