"""Seeded synthetic workloads: shapes, permutations and input values.

This module only *describes* problems (dims, perm, element size, seed) and
draws input values.  It holds none of the transpose arithmetic and is the one
module that both the CPU checker's tests and the GPU path's tests feed from.

Conventions: ``dims[0]`` is the stride-1 dimension; ``perm[j]`` is the input
dimension found at output position ``j``.

The five workload families are synthetic stand-ins, at 2^24..2^26 elements, for
the paper's benchmark shapes: random-extent tensors of ranks 2-7 with 500
permutations per rank (Section 3.1), rank-8/rank-12 tensors with four large and
many small dimensions (Section 3.2) and the contraction sample whose tensors
have a few large leading dimensions and all other extents 8 (Section 3.4).
"""
from __future__ import annotations

import itertools
import math
from dataclasses import dataclass, field
from typing import List, Sequence, Tuple

import numpy as np

SEED_BASE = 170501598 * 1_000_000
LOG2_VOL = 26


@dataclass(frozen=True)
class Case:
    config: int                 # 1..5 = workload family, 0 = ad-hoc test case
    index: int                  # case number inside the family
    dims: Tuple[int, ...]
    perm: Tuple[int, ...]
    elem_size: int              # 4 or 8 bytes
    tag: str = ""
    seed: int = field(default=0)

    @property
    def rank(self) -> int:
        return len(self.dims)

    @property
    def volume(self) -> int:
        return math.prod(self.dims)

    @property
    def bytes_moved(self) -> int:
        """Read + write bytes: 2 * vol * E (bandwidth formula of Section 3.1)."""
        return 2 * self.volume * self.elem_size

    @property
    def name(self) -> str:
        return f"c{self.config}_{self.index:03d}{('_' + self.tag) if self.tag else ''}"


def case_seed(config: int, index: int) -> int:
    return SEED_BASE + 10_000 * config + index


def make_case(config, index, dims, perm, elem_size, tag="") -> Case:
    return Case(config, index, tuple(int(d) for d in dims), tuple(int(p) for p in perm),
                int(elem_size), tag, case_seed(config, index))


# ---------------------------------------------------------------------------
# input values
# ---------------------------------------------------------------------------

def uniform_values(case: Case) -> np.ndarray:
    """Flat input buffer, uniform in [-1, 1), float64 or float32 by element size."""
    rng = np.random.default_rng(case.seed)
    if case.elem_size == 8:
        a = rng.random(case.volume, dtype=np.float64)
        a *= 2.0
        a -= 1.0
        return a
    a = rng.random(case.volume, dtype=np.float32)
    a *= np.float32(2.0)
    a -= np.float32(1.0)
    return a


def stamp_values(case: Case) -> np.ndarray:
    """Index stamp: element i holds the integer i (int64 or int32 by element size)."""
    return np.arange(case.volume, dtype=np.int64 if case.elem_size == 8 else np.int32)


def scrambled_stamp_values(n: int, elem_size: int) -> np.ndarray:
    """n distinct unsigned words of elem_size bytes: element i holds i times an odd constant,
    modulo the word size.  Multiplication by an odd number is a bijection of the words, so the
    values are pairwise different (any two elements that trade places show up in a bit-for-bit
    comparison) and every byte of a word, the high half included, varies from element to
    element."""
    if elem_size == 8:
        return np.arange(n, dtype=np.uint64) * np.uint64(0x9E3779B97F4A7C15)
    return np.arange(n, dtype=np.uint32) * np.uint32(0x9E3779B1)


def bitpattern_values(case: Case) -> np.ndarray:
    """Random raw bit patterns (NaN payloads, -0.0, denormals included) as unsigned ints."""
    rng = np.random.default_rng(case.seed ^ 0x5A5A5A5A)
    dt = np.uint64 if case.elem_size == 8 else np.uint32
    a = rng.integers(0, np.iinfo(dt).max, size=case.volume, dtype=dt, endpoint=True)
    if a.size >= 4:
        if case.elem_size == 8:
            a[:4] = [0x8000000000000000, 0x7FF8000000000001, 0x0000000000000001, 0xFFF0000000000000]
        else:
            a[:4] = [0x80000000, 0x7FC00001, 0x00000001, 0xFF800000]
    return a


def sample_positions(case: Case, n: int) -> np.ndarray:
    """n seeded output scalar positions (first, last and random ones)."""
    rng = np.random.default_rng(case.seed ^ 0x0C0FFEE)
    pos = rng.integers(0, case.volume, size=n, dtype=np.int64)
    pos[0] = 0
    pos[-1] = case.volume - 1
    return pos


# ---------------------------------------------------------------------------
# shape helpers
# ---------------------------------------------------------------------------

def _random_non_identity_perm(rng, r: int) -> Tuple[int, ...]:
    while True:
        p = tuple(int(x) for x in rng.permutation(r))
        if p != tuple(range(r)):
            return p


def _random_dims(rng, r: int, lo: float, hi: float, log2_vol: int = LOG2_VOL,
                 fixed0: int | None = None) -> Tuple[int, ...]:
    """Extents with log2 ~ U[lo, hi], shifted so the logs sum to log2_vol, rounded to
    integers >= 2; the largest extent is then reset so the volume lands within 3 % of
    2^log2_vol.  ``fixed0`` pins dims[0] and rescales the others."""
    target = float(2 ** log2_vol)
    for _ in range(1000):
        logs = rng.uniform(lo, hi, size=r)
        if fixed0 is not None:
            rest = logs[1:]
            rest += (log2_vol - math.log2(fixed0) - rest.sum()) / max(1, r - 1)
            logs = np.concatenate([[math.log2(fixed0)], rest])
        else:
            logs += (log2_vol - logs.sum()) / r
        dims = [max(2, int(round(2.0 ** x))) for x in logs]
        if fixed0 is not None:
            dims[0] = int(fixed0)
        free = range(1, r) if (fixed0 is not None and r > 1) else range(r)
        big = max(free, key=lambda z: dims[z])
        others = math.prod(d for z, d in enumerate(dims) if z != big)
        dims[big] = max(2, int(round(target / others)))
        vol = math.prod(dims)
        if abs(vol - target) <= 0.03 * target:
            return tuple(dims)
    raise RuntimeError("could not draw dims")


# ---------------------------------------------------------------------------
# the five configurations
# ---------------------------------------------------------------------------

def config1() -> List[Case]:
    """Rank-2 fp64 matrix transpose, 2048 x 2048."""
    return [make_case(1, 0, (2048, 2048), (1, 0), 8, "r2")]


def config2() -> List[Case]:
    """Rank-4 fp64, 96^4, all 23 non-identity permutations in lexicographic order."""
    cases = []
    idx = 0
    for p in itertools.permutations(range(4)):
        if p == (0, 1, 2, 3):
            continue
        cases.append(make_case(2, idx, (96, 96, 96, 96), p, 8, "p" + "".join(map(str, p))))
        idx += 1
    return cases


def config3() -> List[Case]:
    """Rank-6 fp64, 20 cases at ~2^26 elements: cases 0-9 have a leading input extent in
    2..8 (packed path), cases 10-19 one in 32..64 (tiled path); random permutations."""
    cases = []
    for i in range(20):
        rng = np.random.default_rng(case_seed(3, i) ^ 0xD1D5)
        d0 = int(rng.integers(2, 9)) if i < 10 else int(rng.integers(32, 65))
        dims = _random_dims(rng, 6, 1.0, 6.0, fixed0=d0)
        perm = _random_non_identity_perm(rng, 6)
        cases.append(make_case(3, i, dims, perm, 8, "small0" if i < 10 else "large0"))
    return cases


def config4(ranks: Sequence[int] = tuple(range(2, 13)), per_rank: int = 30) -> List[Case]:
    """Rank sweep 2..12, fp64, 30 cases per rank at ~2^26 elements.  Cases 0-23: uniformly
    random non-identity permutation; cases 24-29: axis 0 stays first, the tail is a random
    non-identity permutation (rank 2 has only (1,0))."""
    cases = []
    for r in ranks:
        for i in range(per_rank):
            index = (r - 2) * 30 + i
            rng = np.random.default_rng(case_seed(4, index) ^ 0xD1D5)
            dims = _random_dims(rng, r, 1.0, LOG2_VOL / r + 1.0)
            if r == 2:
                perm = (1, 0)
            elif i < 24:
                perm = _random_non_identity_perm(rng, r)
            else:
                tail = _random_non_identity_perm(rng, r - 1)
                perm = (0,) + tuple(t + 1 for t in tail)
            cases.append(make_case(4, index, dims, perm, 8, f"r{r}"))
    return cases


def config5() -> List[Case]:
    """Contraction-feeding fp32 transposes: rank 8 with every extent 8 and rank 6 with
    every extent 16 (2^24 elements each), 40 permutations each that move an index group
    to the front (cases 0-19) or to the back (20-39); the group keeps its order in even
    cases and is shuffled in odd ones."""
    cases = []
    index = 0
    for r, ext in ((8, 8), (6, 16)):
        for i in range(40):
            rng = np.random.default_rng(case_seed(5, index) ^ 0xD1D5)
            while True:
                size = int(rng.integers(1, r))
                group = sorted(int(x) for x in rng.choice(r, size=size, replace=False))
                rest = [z for z in range(r) if z not in group]
                if i % 2 == 1:
                    group = [int(x) for x in rng.permutation(group)]
                perm = tuple(group + rest) if i < 20 else tuple(rest + group)
                if perm != tuple(range(r)):
                    break
            cases.append(make_case(5, index, (ext,) * r, perm, 4,
                                   f"r{r}{'front' if i < 20 else 'back'}"))
            index += 1
    return cases


def all_configs() -> dict:
    return {1: config1(), 2: config2(), 3: config3(), 4: config4(), 5: config5()}


# ---------------------------------------------------------------------------
# further shapes printed in the paper (Section 3.2 and Figure 8)
# ---------------------------------------------------------------------------

SET2_RANK8_DIMS = (5, 3, 2, 4, 35, 33, 37, 40)
SET2_RANK12_DIMS = (2, 3, 4, 3, 2, 2, 3, 2, 20, 18, 22, 24)


def set2(n_random: int = 500) -> List[Case]:
    """Section 3.2 shapes: the printed rank-8 and rank-12 extents with seeded random
    permutations plus the trivial and the reverse one."""
    cases = []
    index = 0
    for dims in (SET2_RANK8_DIMS, SET2_RANK12_DIMS):
        r = len(dims)
        perms = [tuple(range(r)), tuple(reversed(range(r)))]
        rng = np.random.default_rng(case_seed(6, r) ^ 0xD1D5)
        perms += [_random_non_identity_perm(rng, r) for _ in range(n_random)]
        for p in perms:
            cases.append(make_case(6, index, dims, p, 8, f"set2r{r}"))
            index += 1
    return cases


def square_sweep() -> List[Case]:
    """Figure 8 shapes: fp32 square matrices with side 13952..13968."""
    return [make_case(7, s - 13952, (s, s), (1, 0), 4, f"side{s}") for s in range(13952, 13969)]


def heldout(per_cell: int = 2) -> List[Case]:
    """Shapes that no constant of the plan selector was fitted on: ranks 2..12, volumes of
    about 2^25 and 2^27 elements, both element sizes, `per_cell` cases each, extents drawn as in
    the rank sweep but from seeds of their own.  Used to compare the selector's picks with
    measurement-selected plans on shapes it has never seen."""
    cases = []
    index = 0
    for r in range(2, 13):
        for log2_vol in (25, 27):
            for elem in (8, 4):
                for _ in range(per_cell):
                    rng = np.random.default_rng(case_seed(8, index) ^ 0x8E1D0)
                    dims = _random_dims(rng, r, 1.0, log2_vol / r + 1.0, log2_vol=log2_vol)
                    perm = (1, 0) if r == 2 else _random_non_identity_perm(rng, r)
                    cases.append(make_case(8, index, dims, perm, elem, f"r{r}v{log2_vol}e{elem}"))
                    index += 1
    return cases


def even_extents() -> List[Case]:
    """Shapes with "round" extents, as application tensors tend to have: every extent a multiple
    of 2, 4, 8 or 16 elements but not of a whole 128-byte line, or one side line-aligned and the
    other not; ranks 2 and 3, 0.05 to 2 GB, both element sizes, seeded.  The selector's constants
    were fitted on random (mostly odd) extents; this family checks it where pairs of elements,
    sector-aligned pieces and line-aligned rows on one side only all come into play."""
    rng = np.random.default_rng(SEED_BASE + 10_000_000)

    def mult(lo, hi, m, not_m=None):
        while True:
            v = int(rng.integers(lo // m, hi // m + 1)) * m
            if not_m is None or v % not_m != 0:
                return v

    shapes = []
    for elem in (8, 4):
        line = 128 // elem
        granules = (2, 4, 8) if elem == 8 else (4, 8, 16)
        for _ in range(3):
            for g in granules:      # matrices: input rows line-aligned, output rows on a granule of g elements
                shapes.append(((mult(4000, 20000, line), mult(4000, 16000, g, 2 * g)), (1, 0), elem, f"in-aligned-g{g * elem}"))
        for _ in range(2):
            for g in granules:      # the other way round
                shapes.append(((mult(4000, 16000, g, 2 * g), mult(4000, 20000, line)), (1, 0), elem, f"out-aligned-g{g * elem}"))
        for g in granules:          # both sides on the granule
            shapes.append(((mult(4000, 16000, g, 2 * g), mult(4000, 16000, g, 2 * g)), (1, 0), elem, f"both-g{g * elem}"))
        perms = [(2, 0, 1), (1, 0, 2), (2, 1, 0), (1, 2, 0)]
        for i in range(6):          # rank 3, every extent on the granule
            g = granules[i % 3]
            shapes.append(((mult(200, 800, g, 2 * g), mult(200, 800, g, 2 * g), mult(100, 400, g)), perms[i % 4], elem, f"rank3-g{g * elem}"))
        for i in range(4):          # rank 3, leading dimension line-aligned
            g = granules[i % 3]
            shapes.append(((mult(256, 1024, line), mult(200, 800, g, 2 * g), mult(100, 400, g)), perms[i % 4], elem, f"rank3-in-aligned-g{g * elem}"))
    return [make_case(10, i, d, p, e, t) for i, (d, p, e, t) in enumerate(shapes)]


def large_tensors() -> List[Case]:
    """Tensors of 4 GiB and more (byte offsets beyond 32 bits; up to 2^31 - 1 elements): square
    and rank-3 power-of-two shapes, the 96^4 block of the second set seven times over, a ragged
    rank-3 tensor and a matrix with odd sides, in both element sizes.  Not from the paper, whose
    largest tensor is 2.6 GB: sized for a GPU with 288 GB of memory."""
    shapes = [
        ((1 << 15, 1 << 15), (1, 0), 8, "sq32768"),
        ((2048, 2048, 160), (1, 0, 2), 8, "batched"),
        ((2048, 2048, 160), (2, 1, 0), 8, "reverse"),
        ((96, 96, 96, 96, 7), (3, 1, 4, 0, 2), 8, "96^4x7"),
        ((96, 96, 96, 96, 7), (0, 2, 1, 3, 4), 8, "96^4x7keep0"),
        ((1031, 1024, 521), (2, 0, 1), 8, "ragged3"),
        ((1 << 15, 1 << 15), (1, 0), 4, "sq32768"),
        ((40000, 27000), (1, 0), 4, "matrix"),
        ((40001, 27001), (1, 0), 4, "oddmatrix"),
    ]
    return [make_case(9, i, d, p, e, t) for i, (d, p, e, t) in enumerate(shapes)]


def contraction_cases(n_cases: int = 24, target_volume: int = 1 << 24) -> list:
    """Seeded sample of binary tensor contractions D += L * R in the style of the paper's
    contraction benchmark (Section 3.4): tensors of rank up to 8, contracted and uncontracted
    dimensions at random places, a few large dimensions and every other extent 8, sizes scaled
    so that the largest of the three tensors has about `target_volume` elements.

    Each case is a dict: name, seed, d / l / r (label strings, first label = stride-1
    dimension) and extents (label -> extent).  Stands in for the paper's 9306-contraction
    sample, which is not reproduced."""
    rng = np.random.default_rng(SEED_BASE + 8_000_000)
    labels = "abcdefghijklmnop"
    cases = []
    while len(cases) < n_cases:
        nc = int(rng.integers(1, 4))               # contracted dims
        fl = int(rng.integers(1, 5))               # uncontracted dims of L
        fr = int(rng.integers(1, 5))
        if fl + nc > 8 or fr + nc > 8 or fl + fr > 8:
            continue
        ls = labels[:fl]
        rs = labels[fl:fl + fr]
        cs = labels[fl + fr:fl + fr + nc]
        ext = {c: 8 for c in ls + rs + cs}
        # up to two large dims in each group
        large = []
        for grp in (ls, rs, cs):
            k = int(rng.integers(1, min(2, len(grp)) + 1))
            large += list(rng.choice(list(grp), size=k, replace=False))
        for c in large:
            ext[c] = int(rng.integers(16, 97))
        vol = lambda s: int(np.prod([ext[c] for c in s], dtype=np.int64))
        # scale the large extents so that the largest tensor is close to the target
        for _ in range(40):
            big = max(vol(ls + rs), vol(ls + cs), vol(cs + rs))
            if 0.7 * target_volume <= big <= 1.4 * target_volume:
                break
            f = (target_volume / big) ** (1.0 / max(1, len(large)))
            for c in large:
                ext[c] = max(2, min(4096, int(round(ext[c] * f))))
        big = max(vol(ls + rs), vol(ls + cs), vol(cs + rs))
        if not (0.4 * target_volume <= big <= 2.5 * target_volume):
            continue
        shuffle = lambda s: "".join(rng.permutation(list(s)))
        case = {"name": f"k{len(cases):02d}_r{fl + fr}{fl + nc}{fr + nc}", "seed": int(SEED_BASE % (1 << 31)) + len(cases),
                "d": shuffle(ls + rs), "l": shuffle(ls + cs), "r": shuffle(cs + rs), "extents": dict(ext)}
        cases.append(case)
    return cases
