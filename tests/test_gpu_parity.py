"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, bit for bit.

Shapes here are small enough for the oracle to finish in well under a second each, yet span
several tiles and ragged edge tiles in every kernel class.  Transposes move bits, so the
bar is exact equality of the raw bytes.
"""
import itertools
import math

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B
from paper_1705_01598_amd import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")
from gpu_util import np_uint, run_plan, to_device  # noqa: E402


def _check(case, plan, kind="bits", offset=0):
    if kind == "bits":
        a = wl.bitpattern_values(case)
    elif kind == "uniform":
        a = wl.uniform_values(case)
    else:
        a = wl.stamp_values(case)
    a_dev = to_device(a)
    got, guards = run_plan(plan, a_dev, case.volume, case.elem_size, offset)
    ref = np_uint(oracle.transpose(np_uint(a), case.dims, case.perm))
    assert guards, f"{case.name}: wrote outside the output buffer"
    bad = np.nonzero(got != ref)[0]
    assert bad.size == 0, (f"{case.name} dims={case.dims} perm={case.perm}: {bad.size} wrong "
                           f"elements, first at {bad[:5]}; plan={B.info_dict(plan.describe())}")


SHAPES = [
    # (dims, perm)
    ((257, 131), (1, 0)),                       # rank-2, ragged both ways
    ((64, 64), (1, 0)),
    ((9, 7), (1, 0)),                           # the tile-illustration shape of the paper, tiny
    ((1000, 3), (1, 0)),                        # long input dim, tiny output dim
    ((3, 1000), (1, 0)),
    ((70, 45, 33), (2, 1, 0)),
    ((70, 45, 33), (1, 2, 0)),
    ((70, 45, 33), (0, 2, 1)),                  # leading dim kept, long enough for row copy
    ((5, 45, 33, 7), (0, 2, 1, 3)),             # leading dim kept, short: packed
    ((6, 5, 4, 7, 3, 8), (3, 0, 5, 2, 1, 4)),
    ((2, 3, 4, 3, 2, 2, 3, 2, 5, 3), (9, 0, 7, 2, 5, 4, 3, 6, 1, 8)),   # rank 10, tiny extents
    ((4, 3, 2, 2, 3, 2, 2, 3, 2, 2, 3, 2), (11, 10, 9, 8, 7, 6, 5, 4, 3, 2, 1, 0)),  # rank-12 reverse
    ((96, 96, 24), (1, 0, 2)),
    ((33, 1, 17, 1, 19), (4, 1, 2, 3, 0)),      # extent-1 dims in the middle
    ((129, 67, 5), (2, 0, 1)),
    ((8, 8, 8, 8, 8), (1, 3, 0, 2, 4)),         # contraction-style, power-of-two strides
    ((16, 16, 16, 16), (2, 3, 0, 1)),           # fuses to a 256 x 256 matrix transpose
    ((16, 6000), (1, 0)),                       # thin matrix: the tile is one contiguous piece of the input
    ((32, 3000), (1, 0)),
    ((5, 3, 7, 4, 8, 3, 9), (6, 4, 1, 3, 0, 2, 5)),   # input run ends at a dim boundary, next dim has 7 values
    ((17, 7, 15, 45, 7), (3, 2, 0, 4, 1)),
    ((128, 128, 32), (1, 0, 2)),                # line-aligned 8-byte shape: pairs sized by pair slots
]


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("dims,perm", SHAPES[::3])
def test_plans_chosen_by_the_analytical_model_match_oracle(dims, perm, elem):
    """selector = 1: the tile is the one the Section-2.3-style model expects to finish first."""
    case = wl.make_case(0, 31, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, selector=1)
    _check(case, plan)
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("dims,perm", SHAPES)
def test_auto_plan_matches_oracle(dims, perm, elem):
    case = wl.make_case(0, 1, dims, perm, elem)
    plan = B.tperm_plan_create(dims, perm, elem)
    _check(case, plan)
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("kclass", [B.KERNEL_NAIVE, B.KERNEL_TILED, B.KERNEL_PACKED, B.KERNEL_ROWCOPY])
@pytest.mark.parametrize("dims,perm", SHAPES)
def test_forced_class_matches_oracle(dims, perm, kclass, elem):
    case = wl.make_case(0, 2, dims, perm, elem)
    try:
        plan = B.tperm_plan_create_forced(dims, perm, elem, kclass)
    except B.TpermError as e:
        assert e.status == B.ERR_KERNEL      # class not legal for this problem
        pytest.skip("class cannot run this shape")
    assert plan.describe().kernel_class == kclass
    _check(case, plan)
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("kclass", [B.KERNEL_AUTO, B.KERNEL_TILED, B.KERNEL_PACKED])
@pytest.mark.parametrize("dims,perm", SHAPES)
def test_large_tensor_form_matches_oracle(dims, perm, kclass, elem):
    """large = 1: the plan and the kernels that tensors of 4 GiB and more get (every tile
    addresses its pieces from its own origin), on shapes a test can afford."""
    case = wl.make_case(0, 17, dims, perm, elem)
    try:
        plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=kclass, large=1)
    except B.TpermError as e:
        assert e.status == B.ERR_KERNEL and kclass != B.KERNEL_AUTO
        pytest.skip("class cannot run this shape")
    info = plan.describe()
    assert info.large == 1 and info.loads_first == 0
    _check(case, plan, offset=(1 if kclass == B.KERNEL_AUTO else 0))
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("cache_policy", [1, 2, 3, 4])
@pytest.mark.parametrize("dims,perm,m,tin,k,tout", [((257, 131), (1, 0), 1, 64, 1, 48), ((70, 45, 33), (2, 1, 0), 1, 16, 2, 9),
                                                   ((6, 5, 4, 7, 3, 8), (3, 0, 5, 2, 1, 4), 3, 3, 3, 5),
                                                   ((5, 45, 33, 7), (0, 2, 1, 3), 2, 45, 2, 30)])
def test_large_tensor_form_explicit_tiles_and_policies(dims, perm, m, tin, k, tout, cache_policy, elem):
    """The same form with ragged explicit tiles, under each cache policy, with one or two LDS images."""
    case = wl.make_case(0, 18, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=m, tile_in=tin, k=k, tile_out=tout,
                                  cache_policy=cache_policy, lds_buffers=1 + cache_policy % 2, large=1)
    assert plan.describe().large == 1
    _check(case, plan, kind="stamp")
    plan.destroy()


TILES = [
    # dims, perm, m, tile_in, k, tile_out  -> ragged chunks on both split dims
    ((257, 131), (1, 0), 1, 32, 1, 32),
    ((257, 131), (1, 0), 1, 64, 1, 48),
    ((257, 131), (1, 0), 1, 100, 1, 7),
    ((70, 45, 33), (2, 1, 0), 1, 32, 1, 16),
    ((70, 45, 33), (2, 1, 0), 1, 16, 2, 9),
    ((20, 7, 33, 5), (2, 1, 3, 0), 2, 3, 2, 4),
    ((70, 45, 33), (1, 0, 2), 1, 16, 2, 5),
    ((6, 5, 4, 7, 3, 8), (3, 0, 5, 2, 1, 4), 3, 3, 3, 5),
    ((6, 5, 4, 7, 3, 8), (3, 0, 5, 2, 1, 4), 2, 4, 2, 4),
    ((5, 45, 33, 7), (0, 2, 1, 3), 2, 11, 2, 8),
    ((5, 45, 33, 7), (0, 2, 1, 3), 2, 45, 2, 30),
    ((1000, 3), (1, 0), 1, 333, 2, 0),
    ((8, 8, 8, 8, 8), (1, 3, 0, 2, 4), 2, 8, 2, 8),
]


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("grid_mode", [-1, 1, 2, 6])
@pytest.mark.parametrize("dims,perm,m,tin,k,tout", TILES)
def test_explicit_tiles_match_oracle(dims, perm, m, tin, k, tout, grid_mode, elem):
    case = wl.make_case(0, 3, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=m, tile_in=tin,
                                  k=k, tile_out=tout, grid_mode=grid_mode, align_out=1 + abs(grid_mode) % 2)
    _check(case, plan)
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("align_out", [1, 2])
@pytest.mark.parametrize("offset", [0, 1, 5])
@pytest.mark.parametrize("dims,perm", SHAPES)
def test_line_aligned_stores_match_oracle(dims, perm, offset, align_out, elem):
    """Both store modes, with output base pointers at several phases inside a cache line."""
    case = wl.make_case(0, 12, dims, perm, elem)
    try:
        plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=B.KERNEL_PACKED, align_out=align_out,
                                      cache_policy=1 + offset % 4)
    except B.TpermError as e:
        assert e.status == B.ERR_KERNEL
        pytest.skip("no LDS-staged plan for this shape")
    _check(case, plan, offset=offset)


ALIGNED_WINDOW_TILES = [
    # dims, perm, m, tile_in, k, tile_out (tile_out in lines of 128 bytes): misaligned output rows
    ((257, 331), (1, 0), 1, 32, 1, 2),          # several chunks, ragged last window
    ((101, 1003), (1, 0), 1, 16, 1, 4),
    ((70, 45, 333), (2, 1, 0), 1, 16, 1, 2),     # rows from two other dims
    ((7, 9, 400, 3), (2, 0, 1, 3), 2, 9, 1, 1),  # packed input run, one line per chunk
    ((37, 130, 5), (1, 0, 2), 1, 37, 1, 2),      # the shifted dim is the only split dim
    ((64, 200), (1, 0), 1, 64, 1, 1),
]


@pytest.mark.parametrize("large", [0, 1])
@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("offset", [0, 1, 7, 15, 16, 31])
@pytest.mark.parametrize("dims,perm,m,tin,k,lines", ALIGNED_WINDOW_TILES)
def test_line_aligned_windows_match_oracle(dims, perm, m, tin, k, lines, offset, elem, large):
    """Line-aligned output windows (halo on the read side, every row shifted to whole lines),
    with the output base pointer at several phases inside a cache line; large = 1: in the form
    tensors of 4 GiB and more run."""
    case = wl.make_case(0, 21, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, m=m, tile_in=tin, k=k,
                                  tile_out=lines * (128 // elem), align_out=2, cache_policy=1 + offset % 4, large=large)
    assert plan.describe().align_out == 1 and plan.describe().large == large
    _check(case, plan, offset=offset)
    plan.destroy()


PAIR_WINDOW_TILES = [
    # dims, perm, tile_in (even), lines per chunk: 4-byte elements moved in pairs
    ((258, 331), (1, 0), 32, 1),
    ((257, 331), (1, 0), 32, 2),               # odd rows: the last chunk of dim 0 reads singly
    ((101, 1003), (1, 0), 16, 4),
    ((71, 45, 333), (2, 1, 0), 16, 2),
    ((38, 130, 5), (1, 0, 2), 38, 2),          # dim 0 whole (even), the shifted dim alone is split
    ((1001, 999), (1, 0), 64, 2),
    ((5, 7, 301), (2, 0, 1), 4, 1),
]


@pytest.mark.parametrize("large", [0, 1])
@pytest.mark.parametrize("in_offset", [0, 1])
@pytest.mark.parametrize("offset", [0, 1, 2, 7, 16, 31])
@pytest.mark.parametrize("dims,perm,tin,lines", PAIR_WINDOW_TILES)
def test_pair_windows_match_oracle(dims, perm, tin, lines, offset, in_offset, large):
    """Pairs of 4-byte elements inside line-aligned output windows: any phase of the output
    pointer, input pointers aligned to one element only, rows of odd length."""
    case = wl.make_case(0, 25, dims, perm, 4)
    plan = B.tperm_plan_create_ex(dims, perm, 4, m=1, tile_in=tin, k=1, tile_out=32 * lines,
                                  align_out=2, vec2=2, cache_policy=1 + (offset + in_offset) % 4, large=large)
    info = plan.describe()
    assert info.align_out == 1 and info.vec2 == 1 and info.large == large, B.info_dict(info)
    a = wl.bitpattern_values(case)
    buf = torch.empty(case.volume + 64, dtype=torch.int32, device="cuda")
    a_dev = buf[32 + in_offset:32 + in_offset + case.volume]
    a_dev.copy_(to_device(a))
    got, guards = run_plan(plan, a_dev, case.volume, 4, offset)
    assert guards
    assert np.array_equal(got, np_uint(oracle.transpose(np_uint(a), dims, perm)))
    plan.destroy()


@pytest.mark.parametrize("large", [0, 1])
@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("dims,perm", [((5001, 4777), (1, 0)), ((2001, 15, 2003), (2, 1, 0))])
def test_heuristic_picks_aligned_windows_and_matches_oracle(dims, perm, elem, large):
    """Misaligned low-rank transposes: the selector takes the aligned-window form by itself;
    plain execution and accumulation both go through it."""
    case = wl.make_case(0, 22, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, large=large)
    assert plan.describe().align_out == 1 and plan.describe().large == large, B.info_dict(plan.describe())
    assert plan.describe().vec2 == (1 if elem == 4 else 0)
    _check(case, plan, offset=3)
    a = wl.uniform_values(case)
    b = wl.uniform_values(wl.make_case(0, 23, dims, perm, elem)) * 3
    a_dev, b_dev = to_device(a), to_device(b)
    B.tperm_execute_accumulate(plan, a_dev.data_ptr(), b_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = np_uint(b_dev.cpu().numpy())
    ref = np_uint(oracle.transpose_accumulate(a, b, dims, perm))
    assert np.array_equal(got, ref)
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
def test_nontemporal_loads_only_policy(elem):
    """Line-aligned input rows, misaligned output rows: the selector takes nontemporal loads with
    cached stores (policy 4)."""
    dims, perm = (1024, 1001), (1, 0)
    case = wl.make_case(0, 24, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, align_out=1)
    if elem == 8:
        assert plan.describe().cache_policy == 4, B.info_dict(plan.describe())
    else:
        plan.destroy()
        plan = B.tperm_plan_create_ex(dims, perm, elem, align_out=1, cache_policy=4)
    _check(case, plan, offset=1)
    _check(case, plan, offset=0)
    plan.destroy()


def _random_midsize_cases():
    """Seeded shapes of 2-16 M elements, ranks 2-5, ragged extents: large enough for the
    selector to use every form it has (aligned windows, pairs, row copies, big tiles)."""
    rng = np.random.default_rng(20240607)
    cases = []
    while len(cases) < 24:
        r = int(rng.integers(2, 6))
        target = float(rng.uniform(21, 24))
        logs = rng.dirichlet(np.ones(r) * 1.5) * target
        dims = tuple(max(2, int(round(2 ** x)) + int(rng.integers(0, 3))) for x in logs)
        if not (1 << 21) <= math.prod(dims) <= (1 << 24):
            continue
        perm = tuple(int(x) for x in rng.permutation(r))
        if perm == tuple(range(r)):
            continue
        cases.append((dims, perm, int(rng.choice([4, 8])), int(rng.integers(0, 4)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("dims,perm,elem,offset,accumulate", _random_midsize_cases())
def test_random_midsize_shapes(dims, perm, elem, offset, accumulate):
    case = wl.make_case(0, 31, dims, perm, elem)
    plan = B.tperm_plan_create(dims, perm, elem)
    if not accumulate:
        _check(case, plan, offset=offset)
    else:
        a = wl.uniform_values(case)
        b = wl.uniform_values(wl.make_case(0, 32, dims, perm, elem)) * 3
        a_dev, b_dev = to_device(a), to_device(b)
        B.tperm_execute_accumulate(plan, a_dev.data_ptr(), b_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert np.array_equal(np_uint(b_dev.cpu().numpy()), np_uint(oracle.transpose_accumulate(a, b, dims, perm))), \
            B.info_dict(plan.describe())
    plan.destroy()


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("threads", [64, 256])
@pytest.mark.parametrize("lds_buffers", [1, 2])
@pytest.mark.parametrize("dims,perm,m,tin,k,tout", TILES[:8])
def test_workgroup_size_and_lds_buffering(dims, perm, m, tin, k, tout, lds_buffers, threads, elem):
    case = wl.make_case(0, 11, dims, perm, elem)
    try:
        plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=m, tile_in=tin,
                                      k=k, tile_out=tout, threads=threads, lds_buffers=lds_buffers,
                                      cache_policy=1 + (lds_buffers % 2), window_in=4, window_out=3,
                                      loads_first=lds_buffers)
    except B.TpermError as e:
        assert e.status == B.ERR_KERNEL and threads == 64     # tile too large for one wavefront
        pytest.skip("tile does not fit a single-wavefront workgroup")
    _check(case, plan)


@pytest.mark.parametrize("pad", [0, 1, 2, 5])
def test_forced_lds_padding(pad):
    dims, perm = (100, 90), (1, 0)
    case = wl.make_case(0, 4, dims, perm, 8)
    plan = B.tperm_plan_create_ex(dims, perm, 8, kernel_class=B.KERNEL_PACKED, m=1, tile_in=50, k=1,
                                  tile_out=30, lds_pad=pad)
    assert plan.describe().lds_pad == pad
    _check(case, plan)


@pytest.mark.parametrize("elem", [8, 4])
def test_all_rank4_permutations(elem):
    dims = (12, 7, 10, 9)
    for perm in itertools.permutations(range(4)):
        case = wl.make_case(0, 5, dims, perm, elem)
        plan = B.tperm_plan_create(dims, perm, elem)
        _check(case, plan, kind="stamp")
        plan.destroy()


@pytest.mark.parametrize("dims,perm", [((7,), (0,)), ((1,), (0,)), ((1, 1, 1), (2, 0, 1)),
                                       ((5, 1, 3), (0, 1, 2)), ((1000003,), (0,)),
                                       ((4, 6, 5), (0, 1, 2)), ((1, 9, 1), (1, 2, 0))])
@pytest.mark.parametrize("elem", [8, 4])
def test_degenerate_shapes_are_copies(dims, perm, elem):
    case = wl.make_case(0, 6, dims, perm, elem)
    plan = B.tperm_plan_create(dims, perm, elem)
    assert plan.describe().kernel_class == B.KERNEL_COPY
    _check(case, plan)


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("offset", [1, 3])
def test_unaligned_base_pointers(elem, offset):
    """Pointers aligned to the element size only (not to 16 bytes) must still work."""
    for dims, perm in [((257, 131), (1, 0)), ((70, 45, 33), (0, 2, 1)), ((1000,), (0,))]:
        case = wl.make_case(0, 7, dims, perm, elem)
        a = wl.bitpattern_values(case)
        a_pad = np.concatenate([np.zeros(offset, dtype=a.dtype), a])
        a_dev = to_device(a_pad)[offset:]
        plan = B.tperm_plan_create(dims, perm, elem)
        got, guards = run_plan(plan, a_dev, case.volume, elem, offset)
        ref = np_uint(oracle.transpose(a, dims, perm))
        assert guards and np.array_equal(got, ref), (dims, perm, elem, offset)


PAIRED_SHAPES = [
    ((70, 45, 33), (0, 2, 1)),
    ((6, 45, 33, 7), (0, 2, 1, 3)),             # three pairs per row: packed
    ((2, 9, 4, 7, 3, 8), (0, 3, 5, 2, 1, 4)),   # a single pair in front
    ((2050, 37, 5), (0, 2, 1)),                 # long rows: row copy
    ((4, 3, 40, 50), (0, 1, 3, 2)),             # leading dims fuse to an even extent
]


@pytest.mark.parametrize("in_off,out_off", [(0, 0), (1, 0), (0, 1), (1, 1), (2, 2)])
@pytest.mark.parametrize("dims,perm", PAIRED_SHAPES)
def test_paired_four_byte_plans(dims, perm, in_off, out_off):
    """4-byte problems run as 8-byte ones when both pointers allow it, and as given otherwise."""
    case = wl.make_case(0, 8, dims, perm, 4)
    a = wl.bitpattern_values(case)
    a_dev = to_device(np.concatenate([np.zeros(in_off, dtype=a.dtype), a]))[in_off:]
    plan = B.tperm_plan_create(dims, perm, 4)
    assert plan.describe().paired == 1
    got, guards = run_plan(plan, a_dev, case.volume, 4, out_off)
    ref = np_uint(oracle.transpose(a, dims, perm))
    assert guards and np.array_equal(got, ref), (dims, perm, in_off, out_off)
    plan.destroy()


def test_paired_plan_measured_and_accumulate():
    dims, perm = (70, 45, 33), (0, 2, 1)
    case = wl.make_case(0, 9, dims, perm, 4)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    scratch = torch.empty(case.volume, dtype=torch.int32, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    plan = B.tperm_plan_create_measured(dims, perm, 4, a_dev.data_ptr(), scratch.data_ptr(), stream, 12)
    assert plan.describe().paired == 1
    ref = np_uint(oracle.transpose(a, dims, perm))
    for off in (0, 1):
        got, guards = run_plan(plan, a_dev, case.volume, 4, off)
        assert guards and np.array_equal(got, ref)
    # accumulation adds 4-byte floats: the plan's unpaired twin runs
    x = wl.uniform_values(case).astype(np.float32)
    y = wl.uniform_values(wl.make_case(0, 10, dims, perm, 4)).astype(np.float32)
    x_dev = torch.from_numpy(x).cuda()
    y_dev = torch.from_numpy(y.copy()).cuda()
    B.tperm_execute_accumulate(plan, x_dev.data_ptr(), y_dev.data_ptr(), stream)
    torch.cuda.synchronize()
    want = oracle.transpose_accumulate(x, y, dims, perm)
    assert np.array_equal(np_uint(y_dev.cpu().numpy()), np_uint(want))
    plan.destroy()


VEC2_SHAPES = [
    ((258, 130), (1, 0)),                        # ragged chunks on both sides, even extents
    ((64, 64), (1, 0)),
    ((64, 45, 32), (2, 1, 0)),
    ((6, 5, 4, 8, 3, 8), (3, 0, 5, 2, 1, 4)),    # pairs along dims 0 and 3
    ((2, 1000), (1, 0)),                         # a single pair per input row
    ((1000, 2), (1, 0)),
    ((16, 16, 16, 16), (2, 3, 0, 1)),
    ((8, 8, 8, 8, 8), (1, 3, 0, 2, 4)),
]


@pytest.mark.parametrize("elem", [4, 8])
@pytest.mark.parametrize("in_off,out_off", [(0, 0), (1, 0), (0, 1), (2, 2)])
@pytest.mark.parametrize("dims,perm", VEC2_SHAPES)
def test_vec2_plans(dims, perm, in_off, out_off, elem):
    """Transposes move pairs of elements when both pointers are aligned to two elements,
    single elements otherwise; bit-exact either way."""
    case = wl.make_case(0, 13, dims, perm, elem)
    a = wl.bitpattern_values(case)
    a_dev = to_device(np.concatenate([np.zeros(in_off, dtype=a.dtype), a]))[in_off:]
    plan = B.tperm_plan_create(dims, perm, elem)
    if plan.describe().vec2 != 1:
        assert elem == 8          # every shape of the list pairs up with 4-byte elements
        pytest.skip("the tile chosen for 8-byte elements has an odd extent")
    got, guards = run_plan(plan, a_dev, case.volume, elem, out_off)
    ref = np_uint(oracle.transpose(a, dims, perm))
    assert guards and np.array_equal(got, ref), (dims, perm, in_off, out_off)
    plan.destroy()


@pytest.mark.parametrize("dims,perm,tin,tout", [((258, 130), (1, 0), 32, 32), ((258, 130), (1, 0), 100, 6),
                                                ((70, 46, 34), (2, 1, 0), 14, 8), ((20, 7, 34, 6), (2, 1, 3, 0), 4, 10)])
@pytest.mark.parametrize("cache_policy", [1, 2, 3, 4])
@pytest.mark.parametrize("elem", [4, 8])
def test_vec2_explicit_tiles(dims, perm, tin, tout, cache_policy, elem):
    case = wl.make_case(0, 14, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=1, tile_in=tin, k=1,
                                  tile_out=tout, vec2=2, cache_policy=cache_policy)
    assert plan.describe().vec2 == 1
    _check(case, plan)
    # such a plan has no plain twin: unaligned pointers and accumulation are refused
    dt = np.int32 if elem == 4 else np.int64
    a_dev = to_device(np.zeros(case.volume + 1, dtype=dt))
    out = torch.zeros(case.volume + 1, dtype=a_dev.dtype, device="cuda")
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, a_dev.data_ptr() + elem, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert e.value.status == B.ERR_ALIGN
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute_accumulate(plan, a_dev.data_ptr(), out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert e.value.status == B.ERR_KERNEL
    plan.destroy()


def test_uniform_values_and_repeat_execution():
    """Same plan executed several times on different inputs (catches a missing barrier)."""
    dims, perm = (150, 40, 30), (2, 0, 1)
    plan = B.tperm_plan_create(dims, perm, 8)
    for i in range(4):
        case = wl.make_case(0, 100 + i, dims, perm, 8)
        _check(case, plan, kind="uniform")


def test_execute_argument_errors():
    dims, perm = (64, 32), (1, 0)
    plan = B.tperm_plan_create(dims, perm, 8)
    a = torch.zeros(64 * 32 + 8, dtype=torch.int64, device="cuda")
    b = torch.zeros(64 * 32 + 8, dtype=torch.int64, device="cuda")
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, a.data_ptr(), a.data_ptr())
    assert e.value.status == B.ERR_ALIAS
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, a.data_ptr(), a.data_ptr() + 64)       # overlapping ranges
    assert e.value.status == B.ERR_ALIAS
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, a.data_ptr() + 4, b.data_ptr())        # not 8-byte aligned
    assert e.value.status == B.ERR_ALIGN
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, 0, b.data_ptr())
    assert e.value.status == B.ERR_NULL
    B.tperm_execute(plan, a.data_ptr(), b.data_ptr())
    torch.cuda.synchronize()


def test_non_default_stream():
    dims, perm = (257, 131), (1, 0)
    case = wl.make_case(0, 9, dims, perm, 8)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    plan = B.tperm_plan_create(dims, perm, 8)
    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        got, guards = run_plan(plan, a_dev, case.volume, 8)
    assert guards and np.array_equal(got, np_uint(oracle.transpose(a, dims, perm)))


def test_measured_plan_matches_oracle():
    dims, perm = (70, 45, 33), (2, 1, 0)
    case = wl.make_case(0, 10, dims, perm, 8)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    scratch = torch.empty(case.volume, dtype=torch.int64, device="cuda")
    plan = B.tperm_plan_create_measured(dims, perm, 8, a_dev.data_ptr(), scratch.data_ptr(),
                                        torch.cuda.current_stream().cuda_stream, 12)
    got, guards = run_plan(plan, a_dev, case.volume, 8)
    assert guards and np.array_equal(got, np_uint(oracle.transpose(a, dims, perm)))


@pytest.mark.parametrize("elem", [8, 4])
def test_measured_cold_plan_matches_oracle(elem):
    """Measurement-based selection with a scratch buffer swept between the timed runs."""
    dims, perm = (64, 30, 129, 5), (2, 0, 3, 1)
    case = wl.make_case(0, 25, dims, perm, elem)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    out = torch.empty_like(a_dev)
    sweep = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    plan = B.tperm_plan_create_measured_cold(dims, perm, elem, a_dev.data_ptr(), out.data_ptr(), stream,
                                             sweep.data_ptr(), sweep.numel(), 16)
    got, guards = run_plan(plan, a_dev, case.volume, elem)
    assert guards and np.array_equal(got, np_uint(oracle.transpose(np_uint(a), dims, perm)))
    plan.destroy()
    # a scratch that overlaps a tensor, or is not 16-byte aligned, is refused
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_measured_cold(dims, perm, elem, a_dev.data_ptr(), out.data_ptr(), stream,
                                          out.data_ptr() + 64, 4096, 4)
    assert e.value.status == B.ERR_ALIAS
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_measured_cold(dims, perm, elem, a_dev.data_ptr(), out.data_ptr(), stream,
                                          sweep.data_ptr() + 4, 4096, 4)
    assert e.value.status == B.ERR_ALIGN


def test_launches_capture_into_a_hip_graph():
    """A fixed sequence of transposes captured once and replayed: every replay, with eager work
    and synchronisation in between, gives what the eager launches give (the library's launches
    are plain kernel nodes: descriptor by value, no memset nodes)."""
    problems = [((257, 131), (1, 0), 8), ((70, 45, 33), (2, 0, 1), 4), ((1001, 15, 203), (2, 1, 0), 8)]
    plans, ins, outs, cases = [], [], [], []
    for dims, perm, elem in problems:
        case = wl.make_case(0, 26, dims, perm, elem)
        cases.append(case)
        plans.append(B.tperm_plan_create(dims, perm, elem))
        ins.append(to_device(wl.bitpattern_values(case)))
        outs.append(torch.zeros_like(ins[-1]))
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for p, a, b in zip(plans, ins, outs):         # first use outside the capture
            B.tperm_execute(p, a.data_ptr(), b.data_ptr(), side.cuda_stream)
    side.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for p, a, b in zip(plans, ins, outs):
            B.tperm_execute(p, a.data_ptr(), b.data_ptr(), torch.cuda.current_stream().cuda_stream)
    for replay in range(3):
        for i, case in enumerate(cases):               # new input bits, stale output, eagerly
            ins[i].copy_(to_device(wl.bitpattern_values(wl.make_case(0, 27 + replay, case.dims, case.perm, case.elem_size))))
            outs[i].zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for i, case in enumerate(cases):
            a = np_uint(ins[i].cpu().numpy())
            ref = np_uint(oracle.transpose(a, case.dims, case.perm))
            assert np.array_equal(np_uint(outs[i].cpu().numpy()), ref), (replay, case.dims)
    for p in plans:
        p.destroy()


def test_copy_bytes():
    n = 1 << 20
    a = torch.arange(n + 3, dtype=torch.int32, device="cuda")
    b = torch.zeros(n + 3, dtype=torch.int32, device="cuda")
    B.tperm_copy_bytes(a.data_ptr(), b.data_ptr(), (n + 3) * 4, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("kclass", [B.KERNEL_AUTO, B.KERNEL_NAIVE, B.KERNEL_PACKED, B.KERNEL_ROWCOPY])
@pytest.mark.parametrize("dims,perm", SHAPES + [((4, 6, 5), (0, 1, 2)), ((1000003,), (0,))])
def test_accumulate_matches_oracle(dims, perm, kclass, elem):
    """out = out + transpose(in): one IEEE addition per element, so still bit-exact."""
    case = wl.make_case(0, 13, dims, perm, elem)
    try:
        plan = B.tperm_plan_create_ex(dims, perm, elem, kernel_class=kclass)
    except B.TpermError as e:
        assert e.status == B.ERR_KERNEL
        pytest.skip("class cannot run this shape")
    a = wl.uniform_values(case)
    b = wl.uniform_values(wl.make_case(0, 14, dims, perm, elem)) * 3
    a_dev, b_dev = to_device(a), to_device(b)
    B.tperm_execute_accumulate(plan, a_dev.data_ptr(), b_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = np_uint(b_dev.cpu().numpy())
    ref = np_uint(oracle.transpose_accumulate(a, b, dims, perm))
    bad = np.nonzero(got != ref)[0]
    assert bad.size == 0, (dims, perm, elem, kclass, bad[:5])


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("dims,perm", SHAPES[::2])
def test_large_tensor_form_accumulates(dims, perm, elem):
    case = wl.make_case(0, 19, dims, perm, elem)
    plan = B.tperm_plan_create_ex(dims, perm, elem, large=1)
    a = wl.uniform_values(case)
    b = wl.uniform_values(wl.make_case(0, 20, dims, perm, elem)) * 3
    a_dev, b_dev = to_device(a), to_device(b)
    B.tperm_execute_accumulate(plan, a_dev.data_ptr(), b_dev.data_ptr(), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    got = np_uint(b_dev.cpu().numpy())
    ref = np_uint(oracle.transpose_accumulate(a, b, dims, perm))
    assert np.array_equal(got, ref), (dims, perm, elem)


def test_cached_one_call_interface():
    """tperm_transpose / tperm_cache_tune / tperm_transpose_accumulate through the plan cache."""
    from gpu_util import GuardedOut
    B.tperm_cache_clear()
    stream = torch.cuda.current_stream().cuda_stream
    problems = [((70, 45, 33), (2, 1, 0), 8), ((70, 45, 33), (0, 2, 1), 4), ((257, 131), (1, 0), 4),
                ((6, 5, 4, 7, 3, 8), (3, 0, 5, 2, 1, 4), 8), ((4, 6, 5), (0, 1, 2), 8)]
    for rep in range(2):
        for i, (dims, perm, elem) in enumerate(problems):
            case = wl.make_case(0, 40 + i + 10 * rep, dims, perm, elem)
            a = wl.bitpattern_values(case)
            a_dev = to_device(a)
            out = GuardedOut(case.volume, elem)
            B.tperm_transpose(dims, perm, elem, a_dev.data_ptr(), out.ptr, stream)
            torch.cuda.synchronize()
            got = np_uint(out.view().cpu().numpy())
            assert out.guards_intact() and np.array_equal(got, np_uint(oracle.transpose(a, dims, perm)))
    s = B.tperm_cache_stats()
    assert s["entries"] == len(problems) and s["misses"] == len(problems) and s["hits"] == len(problems)
    # tuning replaces the cached plan; results stay bit-exact
    dims, perm, elem = problems[0]
    case = wl.make_case(0, 77, dims, perm, elem)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    scratch = torch.empty(case.volume, dtype=torch.int64, device="cuda")
    B.tperm_cache_tune(dims, perm, elem, a_dev.data_ptr(), scratch.data_ptr(), stream)
    assert B.tperm_cache_stats()["entries"] == len(problems)
    out = GuardedOut(case.volume, elem)
    B.tperm_transpose(dims, perm, elem, a_dev.data_ptr(), out.ptr, stream)
    torch.cuda.synchronize()
    ref = oracle.transpose(a, dims, perm)
    assert out.guards_intact() and np.array_equal(np_uint(out.view().cpu().numpy()), np_uint(ref))
    assert np.array_equal(np_uint(scratch.cpu().numpy()), np_uint(ref))   # the timed runs wrote it too
    # accumulate through the cache
    x = wl.uniform_values(case)
    y = wl.uniform_values(wl.make_case(0, 78, dims, perm, elem))
    x_dev, y_dev = torch.from_numpy(x).cuda(), torch.from_numpy(y.copy()).cuda()
    B.tperm_transpose(dims, perm, elem, x_dev.data_ptr(), y_dev.data_ptr(), stream, accumulate=True)
    torch.cuda.synchronize()
    assert np.array_equal(np_uint(y_dev.cpu().numpy()), np_uint(oracle.transpose_accumulate(x, y, dims, perm)))
    # errors pass through
    with pytest.raises(B.TpermError) as e:
        B.tperm_transpose(dims, perm, elem, a_dev.data_ptr(), a_dev.data_ptr(), stream)
    assert e.value.status == B.ERR_ALIAS
    B.tperm_cache_clear()
    assert B.tperm_cache_stats()["entries"] == 0
