"""GPU parity at the full benchmark sizes, with the plans the benchmark times.

Every case of every workload family is compared with the CPU oracle element by element, bit
for bit, over the whole tensor: the 2048^2 matrix, all 23 permutations of the 96^4 tensor, the
20 rank-6 cases, the 330 cases of the rank sweep, the 80 contraction-feeding cases, the printed
rank-8 / rank-12 shapes of Section 3.2 and the square matrices of Figure 8.

Input values are distinct scrambled index stamps (element i holds i times an odd 64- or 32-bit
constant): no two elements are equal, so elements that trade places cannot hide, and the high
half of every word carries information, so a mix-up inside 8- or 16-byte accesses cannot
either.  A subset is repeated with the values the workloads are defined with (uniform in
[-1, 1) from the case's seed) and with raw random bit patterns.  The output buffer is
pre-filled with a sentinel and fenced by guard bands: an element never written, or anything
written outside the tensor, fails the comparison too.
"""
import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B
from paper_1705_01598_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
from gpu_util import GUARD, np_uint, to_device  # noqa: E402

SENT = -1  # all bits set


def _stream():
    return torch.cuda.current_stream().cuda_stream


class _Arena:
    """Scrambled-stamp input on host and device, plus a guarded output buffer, per element
    size; grown to the largest volume asked for and reused by every case (a case of volume v
    takes the first v stamps)."""

    def __init__(self):
        self.host = {}
        self.dev = {}
        self.out = {}

    def get(self, volume, elem):
        if elem not in self.host or self.host[elem].size < volume:
            self.dev.pop(elem, None)
            self.out.pop(elem, None)
            torch.cuda.empty_cache()
            h = wl.scrambled_stamp_values(volume, elem)
            assert not bool((h == np_uint(np.array([SENT], dtype=np.int64 if elem == 8 else np.int32))[0]).any())
            self.host[elem] = h
            self.dev[elem] = to_device(h)
            self.out[elem] = torch.empty(volume + 2 * GUARD, dtype=self.dev[elem].dtype, device="cuda")
        return self.host[elem][:volume], self.dev[elem][:volume], self.out[elem][:volume + 2 * GUARD]


_arena = _Arena()


def _assert_equal_to_oracle(out, ref_bits, case, plan):
    """out: guarded device buffer; ref_bits: expected tensor as unsigned host words."""
    vol = case.volume
    desc = f"{case.name} dims={case.dims} perm={case.perm} plan={B.info_dict(plan.describe())}"
    ref_dev = to_device(ref_bits)
    body = out[GUARD:GUARD + vol]
    if not torch.equal(body, ref_dev):
        bad = torch.nonzero(body != ref_dev).flatten()
        first = [int(x) for x in bad[:4].cpu()]
        raise AssertionError(f"{desc}: {bad.numel()} of {vol} elements differ from the oracle, first at {first}")
    assert bool((out[:GUARD] == SENT).all()) and bool((out[GUARD + vol:] == SENT).all()), \
        "written outside the tensor: " + desc


def _full_stamp_compare(case, plan=None):
    """Whole-tensor, bit-for-bit comparison of one case on scrambled-stamp input."""
    a, a_dev, out = _arena.get(case.volume, case.elem_size)
    plan = plan or B.tperm_plan_create(case.dims, case.perm, case.elem_size)
    out.fill_(SENT)
    B.tperm_execute(plan, a_dev.data_ptr(), out.data_ptr() + GUARD * case.elem_size, _stream())
    torch.cuda.synchronize()
    _assert_equal_to_oracle(out, oracle.transpose(a, case.dims, case.perm), case, plan)


def _full_compare(case, values="uniform"):
    """The same on the workload's own values (uniform in [-1, 1)) or raw random bits."""
    a = wl.uniform_values(case) if values == "uniform" else wl.bitpattern_values(case)
    a_dev = to_device(a)
    out = torch.full((case.volume + 2 * GUARD,), SENT, dtype=a_dev.dtype, device="cuda")
    plan = B.tperm_plan_create(case.dims, case.perm, case.elem_size)
    B.tperm_execute(plan, a_dev.data_ptr(), out.data_ptr() + GUARD * case.elem_size, _stream())
    torch.cuda.synchronize()
    _assert_equal_to_oracle(out, np_uint(oracle.transpose(np_uint(a), case.dims, case.perm)), case, plan)


# --- config 1: 2048 x 2048 fp64 ------------------------------------------------------------

def test_config1_full():
    _full_compare(wl.config1()[0])
    _full_stamp_compare(wl.config1()[0])


# --- config 2: 96^4 fp64, all 23 non-identity permutations -----------------------------------

@pytest.mark.parametrize("idx", range(23))
def test_config2_every_permutation_full(idx):
    _full_stamp_compare(wl.config2()[idx])


@pytest.mark.parametrize("idx", [0, 1, 8, 15, 22])
def test_config2_uniform_values_full(idx):
    _full_compare(wl.config2()[idx])


# --- config 3: rank 6 fp64, 20 cases --------------------------------------------------------

@pytest.mark.parametrize("idx", range(20))
def test_config3_every_case_full(idx):
    _full_stamp_compare(wl.config3()[idx])


@pytest.mark.parametrize("idx", [1, 16])
def test_config3_random_bits_full(idx):
    _full_compare(wl.config3()[idx], values="bits")


# --- config 4: rank sweep 2..12, 30 cases per rank ------------------------------------------

@pytest.mark.parametrize("rank", list(range(2, 13)))
def test_config4_rank_sweep_every_case_full(rank):
    for case in wl.config4(ranks=(rank,)):
        _full_stamp_compare(case)


@pytest.mark.parametrize("idx", [40, 171, 300, 329])
def test_config4_uniform_values_full(idx):
    _full_compare(wl.config4()[idx])


# --- config 5: fp32 contraction-feeding transposes, 80 cases --------------------------------

def test_config5_all_cases_full_compare():
    for case in wl.config5():
        _full_stamp_compare(case)
        _full_compare(case, values="uniform" if case.index % 2 else "bits")


# --- plans chosen by measurement, accumulation, concurrency ---------------------------------

def test_measured_plans_on_config2_subset():
    """Measurement-based selection (Section 2.3) returns a plan that is still exact."""
    for case in wl.config2()[::11]:
        a, a_dev, out = _arena.get(case.volume, 8)
        plan = B.tperm_plan_create_measured(case.dims, case.perm, 8, a_dev.data_ptr(),
                                            out.data_ptr() + GUARD * 8, _stream(), 16)
        _full_stamp_compare(case, plan)


def test_accumulate_full_size():
    """out = out + transpose(in) on two C2 permutations, element by element."""
    for case in (wl.config2()[3], wl.config2()[22]):
        a = wl.uniform_values(case)
        b = wl.uniform_values(wl.make_case(2, 100 + case.index, case.dims, case.perm, 8))
        a_dev, b_dev = to_device(a), to_device(b)
        plan = B.tperm_plan_create(case.dims, case.perm, 8)
        B.tperm_execute_accumulate(plan, a_dev.data_ptr(), b_dev.data_ptr(), _stream())
        torch.cuda.synchronize()
        got = np_uint(b_dev.cpu().numpy())
        ref = np_uint(oracle.transpose_accumulate(a, b, case.dims, case.perm))
        assert np.array_equal(got, ref), case.name


def test_two_streams_share_one_plan():
    """A plan is immutable: the same plan executed concurrently on two streams."""
    case = wl.config3()[5]
    plan = B.tperm_plan_create(case.dims, case.perm, 8)
    a, a_dev, _ = _arena.get(case.volume, 8)
    outs = [torch.full((case.volume,), SENT, dtype=torch.int64, device="cuda") for _ in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for rep in range(3):
        for s, o in zip(streams, outs):
            B.tperm_execute(plan, a_dev.data_ptr(), o.data_ptr(), s.cuda_stream)
    torch.cuda.synchronize()
    ref_dev = to_device(oracle.transpose(a, case.dims, case.perm))
    assert torch.equal(outs[0], ref_dev) and torch.equal(outs[1], ref_dev)


# --- shapes printed in the paper -------------------------------------------------------------

@pytest.mark.parametrize("which", [0, 1])
def test_paper_set2_shapes_full(which):
    """The rank-8 (205 M elements) and rank-12 (328 M elements, 2.6 GB: byte offsets beyond
    2^31) shapes printed in Section 3.2, with the trivial, the reverse and seeded random
    permutations, every element compared."""
    for case in [c for c in wl.set2(6) if c.rank == (8, 12)[which]]:
        _full_stamp_compare(case)


@pytest.mark.parametrize("side", [13952, 13953, 13966, 13967])
def test_figure8_squares_full(side):
    """The square 4-byte matrices of the alignment sweep (Section 3.1, Figure 8): whole lines
    per row, and rows that start anywhere in a line (pairs inside line-aligned windows; odd
    sides end every input row with a single element)."""
    _full_stamp_compare(next(c for c in wl.square_sweep() if c.dims[0] == side))


# --- tensors of 4 GiB and more ----------------------------------------------------------------

BIG_CASES = [
    # dims, perm, element size, forced class (None = the selector's plan)
    ((1031, 1024, 521), (2, 0, 1), 8, None),      # 4.40 GB, ragged, rank 3
    ((40000, 27000), (1, 0), 4, None),            # 4.32 GB of 4-byte elements, a plain matrix transpose
    ((96, 96, 96, 96, 7), (3, 1, 4, 0, 2), 8, None),   # 4.76 GB, the 96^4 block seven times over
    ((1031, 1024, 521), (1, 2, 0), 8, "naive"),   # the gather kernel, which such tensors fall back to
]


@pytest.mark.parametrize("dims,perm,elem,forced", BIG_CASES)
def test_tensors_beyond_4_gib_full(dims, perm, elem, forced):
    """Byte offsets beyond 2^32: every tile addresses its pieces from its own origin (the plan
    reports large = 1).  Whole-tensor comparison with the oracle on scrambled index stamps,
    sentinel pre-fill and guard bands as everywhere else; then the accumulating form on the
    same plan (out = out + transposed in, with integer-valued doubles / floats so that the one
    addition per element is exact and cheap to predict from the first result)."""
    case = wl.make_case(9, 0, dims, perm, elem)
    assert case.volume * elem >= (1 << 32)
    plan = (B.tperm_plan_create_forced(dims, perm, elem, B.KERNEL_NAIVE) if forced == "naive"
            else B.tperm_plan_create(dims, perm, elem))
    info = plan.describe()
    assert info.large == 1
    if forced is None:
        assert info.kernel_class in (B.KERNEL_TILED, B.KERNEL_PACKED)
    a = wl.scrambled_stamp_values(case.volume, elem)
    a_dev = to_device(a)
    out = torch.full((case.volume + 2 * GUARD,), SENT, dtype=a_dev.dtype, device="cuda")
    B.tperm_execute(plan, a_dev.data_ptr(), out.data_ptr() + GUARD * elem, _stream())
    torch.cuda.synchronize()
    ref = oracle.transpose(a, dims, perm)
    _assert_equal_to_oracle(out, ref, case, plan)
    if len(dims) == 5:
        # a plan chosen by timing candidates (Section 2.3) on such a tensor: same bar
        measured = B.tperm_plan_create_measured(dims, perm, elem, a_dev.data_ptr(), out.data_ptr() + GUARD * elem, _stream(), 6)
        assert measured.describe().large == 1
        out.fill_(SENT)
        B.tperm_execute(measured, a_dev.data_ptr(), out.data_ptr() + GUARD * elem, _stream())
        torch.cuda.synchronize()
        _assert_equal_to_oracle(out, ref, case, measured)
    del a_dev, out
    torch.cuda.empty_cache()
    if forced is None:
        # accumulate: in = small integers as floating point, out starts at 1.0 everywhere
        ftype = np.float64 if elem == 8 else np.float32
        small = (np.arange(case.volume, dtype=np.int64) % 1021).astype(ftype)
        in_dev = to_device(small)
        acc = torch.ones(case.volume, dtype=torch.float64 if elem == 8 else torch.float32, device="cuda")
        B.tperm_execute_accumulate(plan, in_dev.data_ptr(), acc.data_ptr(), _stream())
        torch.cuda.synchronize()
        expect = to_device(oracle.transpose(small, dims, perm)).view(acc.dtype) + 1.0
        assert torch.equal(acc, expect), f"accumulate on {dims} {perm}"
        del in_dev, acc, expect
    del a, ref
    torch.cuda.empty_cache()
