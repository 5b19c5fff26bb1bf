"""Tensor contraction D += L * R through transposes and one GEMM (application layer).

The use the paper makes of its transpose library (Section 3.4: the indirect, "transpose -
transpose - GEMM - transpose" implementation of a binary tensor contraction): the left input is
brought to the layout (uncontracted dims, contracted dims), the right input to (contracted dims,
uncontracted dims), one matrix product gives the result in the layout (left uncontracted, right
uncontracted), and a last transpose accumulates it into the destination.  The three transposes
run through the tperm library (the last one with ``tperm_transpose_accumulate``); the matrix
product is the vendor GEMM reached through ``torch.mm`` (hipBLASLt / rocBLAS).  Everything here
is argument bookkeeping around those two.

Conventions as everywhere in this package: a tensor is a flat buffer, the FIRST label / extent
is the stride-1 dimension.  A contraction is given by three label strings, e.g.
``D="abef", L="abcd", R="cdef"``: labels shared by L and R and absent from D are summed over; every
other label must occur in D and in exactly one of L, R.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Dict, List, Sequence, Tuple


@dataclass(frozen=True)
class ContractionLayout:
    """Index bookkeeping of one contraction (pure host logic, no GPU needed)."""
    d_labels: str
    l_labels: str
    r_labels: str
    extents: Tuple[Tuple[str, int], ...]
    free_l: str          # uncontracted labels of L, in D's order
    free_r: str          # uncontracted labels of R, in D's order
    summed: str          # contracted labels, in L's order
    l_perm: Tuple[int, ...]   # gather permutation L -> (free_l, summed)
    r_perm: Tuple[int, ...]   # gather permutation R -> (summed, free_r)
    t_perm: Tuple[int, ...]   # gather permutation (free_l, free_r) -> D
    m: int
    n: int
    k: int

    def dims(self, labels: str) -> Tuple[int, ...]:
        e = dict(self.extents)
        return tuple(e[c] for c in labels)

    @property
    def flops(self) -> int:
        return 2 * self.m * self.n * self.k

    @property
    def arithmetic_intensity(self) -> float:
        """2 sqrt(vol(D) vol(L) vol(R)) / (vol(D) + vol(L) + vol(R)), the paper's measure."""
        vd, vl, vr = self.m * self.n, self.m * self.k, self.k * self.n
        return 2.0 * math.sqrt(float(vd) * vl * vr) / (vd + vl + vr)


def layout(d_labels: str, l_labels: str, r_labels: str, extents: Dict[str, int]) -> ContractionLayout:
    """Work out which labels are summed and the three gather permutations."""
    for s in (d_labels, l_labels, r_labels):
        if len(set(s)) != len(s):
            raise ValueError(f"repeated label in '{s}'")
        for c in s:
            if c not in extents or int(extents[c]) < 1:
                raise ValueError(f"label '{c}' has no positive extent")
    summed = "".join(c for c in l_labels if c in r_labels)
    if any(c in d_labels for c in summed):
        raise ValueError("a label shared by both inputs must not occur in the result")
    free_l = "".join(c for c in d_labels if c in l_labels)
    free_r = "".join(c for c in d_labels if c in r_labels)
    if len(free_l) + len(free_r) != len(d_labels):
        raise ValueError("every result label must come from exactly one input")
    if set(free_l) | set(summed) != set(l_labels) or set(free_r) | set(summed) != set(r_labels):
        raise ValueError("every input label must be summed or occur in the result")
    if not summed:
        raise ValueError("nothing to sum over")
    l_target, r_target, t_labels = free_l + summed, summed + free_r, free_l + free_r
    e = {c: int(extents[c]) for c in set(d_labels + l_labels + r_labels)}
    prod = lambda s: math.prod(e[c] for c in s)
    return ContractionLayout(
        d_labels, l_labels, r_labels, tuple(sorted(e.items())), free_l, free_r, summed,
        tuple(l_labels.index(c) for c in l_target), tuple(r_labels.index(c) for c in r_target),
        tuple(t_labels.index(c) for c in d_labels), prod(free_l), prod(free_r), prod(summed))


class Contraction:
    """A planned contraction: three cached-plan transposes, one GEMM, workspace included."""

    def __init__(self, d_labels: str, l_labels: str, r_labels: str, extents: Dict[str, int], dtype, device="cuda"):
        import torch
        from . import binding as B
        self._torch, self._B = torch, B
        self.lay = layout(d_labels, l_labels, r_labels, extents)
        if dtype not in (torch.float32, torch.float64):
            raise ValueError("float32 or float64 only")
        self.dtype = dtype
        self.elem = 4 if dtype == torch.float32 else 8
        lay = self.lay
        ident = lambda p: tuple(p) == tuple(range(len(p)))
        # inputs already in matrix layout are used in place
        self._lp = None if ident(lay.l_perm) else torch.empty(lay.m * lay.k, dtype=dtype, device=device)
        self._rp = None if ident(lay.r_perm) else torch.empty(lay.k * lay.n, dtype=dtype, device=device)
        self._t = torch.empty(lay.m * lay.n, dtype=dtype, device=device)

    def run(self, l, r, d, timings: dict = None) -> None:
        """d += l * r; all three are flat device tensors of the contraction's dtype."""
        torch, B, lay = self._torch, self._B, self.lay
        for t, labels in ((l, lay.l_labels), (r, lay.r_labels), (d, lay.d_labels)):
            if t.dtype != self.dtype or t.numel() != math.prod(lay.dims(labels)) or not t.is_contiguous():
                raise ValueError("operand does not match the planned contraction")
        stream = torch.cuda.current_stream().cuda_stream
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(5)] if timings is not None else None
        mark = (lambda i: ev[i].record()) if ev else (lambda i: None)
        mark(0)
        lp, rp = l, r
        if self._lp is not None:
            B.tperm_transpose(lay.dims(lay.l_labels), lay.l_perm, self.elem, l.data_ptr(), self._lp.data_ptr(), stream)
            lp = self._lp
        mark(1)
        if self._rp is not None:
            B.tperm_transpose(lay.dims(lay.r_labels), lay.r_perm, self.elem, r.data_ptr(), self._rp.data_ptr(), stream)
            rp = self._rp
        mark(2)
        # column-major (m x k)(k x n) = (m x n)  is  row-major (n x k)(k x m) = (n x m)
        torch.mm(rp.view(lay.n, lay.k), lp.view(lay.k, lay.m), out=self._t.view(lay.n, lay.m))
        mark(3)
        t_dims = lay.dims(lay.free_l + lay.free_r)
        B.tperm_transpose(t_dims, lay.t_perm, self.elem, self._t.data_ptr(), d.data_ptr(), stream, accumulate=True)
        mark(4)
        if ev:
            ev[4].synchronize()
            names = ("transpose_l_ms", "transpose_r_ms", "gemm_ms", "transpose_d_ms")
            for i, name in enumerate(names):
                timings[name] = ev[i].elapsed_time(ev[i + 1])
            timings["total_ms"] = ev[0].elapsed_time(ev[4])


def contract(d_labels: str, l_labels: str, r_labels: str, extents: Dict[str, int], l, r, d) -> None:
    """One-shot d += l * r (plans and workspace are built on every call; keep a Contraction
    object around when the same contraction repeats)."""
    Contraction(d_labels, l_labels, r_labels, extents, d.dtype, d.device).run(l, r, d)


def _bench(argv: Sequence[str] = None) -> None:
    """Times the seeded contraction sample: GFLOP/s and the share of time spent transposing,
    against arithmetic intensity.  One JSON line per case, then a summary line."""
    import argparse
    import json
    import numpy as np
    import torch
    from . import workloads as wl
    ap = argparse.ArgumentParser(description=_bench.__doc__)
    ap.add_argument("--dtype", choices=["f32", "f64"], default="f64")
    ap.add_argument("--reps", type=int, default=5)
    args = ap.parse_args(argv)
    dtype = torch.float64 if args.dtype == "f64" else torch.float32
    rows = []
    for case in wl.contraction_cases():
        c = Contraction(case["d"], case["l"], case["r"], case["extents"], dtype)
        lay = c.lay
        g = torch.Generator(device="cuda").manual_seed(case["seed"])
        l = torch.rand(lay.m * lay.k, dtype=dtype, device="cuda", generator=g) * 2 - 1
        r = torch.rand(lay.k * lay.n, dtype=dtype, device="cuda", generator=g) * 2 - 1
        d = torch.zeros(lay.m * lay.n, dtype=dtype, device="cuda")
        c.run(l, r, d)
        best = None
        for _ in range(args.reps):
            t = {}
            c.run(l, r, d, t)
            if best is None or t["total_ms"] < best["total_ms"]:
                best = t
        tr = best["transpose_l_ms"] + best["transpose_r_ms"] + best["transpose_d_ms"]
        row = {"case": case["name"], "d": case["d"], "l": case["l"], "r": case["r"], "m": lay.m, "n": lay.n, "k": lay.k,
               "arithmetic_intensity": round(lay.arithmetic_intensity, 1),
               "gflops": round(lay.flops / best["total_ms"] / 1e6, 1),
               "gemm_gflops": round(lay.flops / best["gemm_ms"] / 1e6, 1),
               "transpose_share": round(tr / best["total_ms"], 4), **{k: round(v, 4) for k, v in best.items()}}
        rows.append(row)
        print(json.dumps(row), flush=True)
    by = sorted(rows, key=lambda x: x["arithmetic_intensity"])
    third = max(1, len(by) // 3)
    summary = {"metric": "tensor contraction through transposes + GEMM", "dtype": args.dtype, "cases": len(rows),
               "low_ai": {"ai_max": by[third - 1]["arithmetic_intensity"],
                          "median_transpose_share": float(np.median([x["transpose_share"] for x in by[:third]]))},
               "high_ai": {"ai_min": by[-third]["arithmetic_intensity"],
                           "median_transpose_share": float(np.median([x["transpose_share"] for x in by[-third:]])),
                           "median_gflops": float(np.median([x["gflops"] for x in by[-third:]]))}}
    print(json.dumps(summary), flush=True)


if __name__ == "__main__":
    _bench()
