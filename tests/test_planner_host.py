"""Host-only tests of the library: C-ABI exports, argument validation, canonical form, the
multiply-shift division, and -- for every plan the GPU tests execute and many more -- the
plan's index maps, evaluated on the CPU with the very arithmetic the kernel runs, against
the oracle's map.  No GPU is needed: plan creation never touches the device."""
import ctypes
import itertools
import math
import os
import re

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B
from paper_1705_01598_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("header,exports", [("tperm.h", "EXPORTS"), ("tperm_tuning.h", "TUNING_EXPORTS")])
def test_library_exports_every_declared_symbol(header, exports):
    """Both headers: every function they declare is bound and exported, and nothing else."""
    text = open(os.path.join(ROOT, "include", header)).read()
    declared = set(re.findall(r"\b(tperm_[a-z_]+)\s*\(", text))
    assert declared == set(getattr(B, exports))
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_product_header_is_the_small_boundary():
    """The product header holds the plan / execute / describe / destroy calls, the measured
    and cached forms and the copy; overrides and self-check hooks live in the tuning header."""
    text = open(os.path.join(ROOT, "include", "tperm.h")).read()
    assert "tperm_plan_opts_t" not in text and "tperm_plan_index_map" not in text
    for name in ("tperm_plan_create", "tperm_plan_create_forced", "tperm_execute", "tperm_execute_accumulate",
                 "tperm_plan_describe", "tperm_plan_destroy", "tperm_status_string"):
        assert re.search(r"\b" + name + r"\s*\(", text), name


def test_forced_create_is_the_options_path_with_a_class():
    for kc in (B.KERNEL_AUTO, B.KERNEL_TILED, B.KERNEL_PACKED, B.KERNEL_NAIVE):
        a = B.info_dict(B.tperm_plan_create_forced((40, 9, 33), (2, 0, 1), 8, kc).describe())
        b = B.info_dict(B.tperm_plan_create_ex((40, 9, 33), (2, 0, 1), 8, kernel_class=kc).describe())
        assert a == b
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_forced((8, 9, 10), (2, 1, 0), 8, B.KERNEL_ROWCOPY)
    assert e.value.status == B.ERR_KERNEL


def test_describe_reports_the_policy_that_is_launched():
    """Variants that are not instantiated fall back to another cache policy; describe() names
    the one that runs."""
    d = lambda **kw: B.tperm_plan_create_ex((64, 40, 64), (2, 1, 0), 8, **kw).describe()
    assert d(cache_policy=4, loads_first=1).cache_policy == 4
    assert d(cache_policy=4, loads_first=2).cache_policy == 1      # nontemporal loads alone: stores-first kernels only
    assert d(cache_policy=3, threads=64).cache_policy == 2          # 64-thread kernels: cached or fully nontemporal
    assert d(cache_policy=4, threads=64).cache_policy == 1
    for pol in (1, 2, 3):
        assert d(cache_policy=pol).cache_policy == pol


def test_status_strings():
    for s in range(13):
        assert B.status_string(s) and B.status_string(s) != "unknown status"
    assert B.status_string(99) == "unknown status"


@pytest.mark.parametrize("dims,perm,elem,status", [
    ((2, 3), (0, 0), 8, B.ERR_PERM),
    ((2, 3), (0, 2), 8, B.ERR_PERM),
    ((2, 3), (-1, 0), 8, B.ERR_PERM),
    ((2, 0), (0, 1), 8, B.ERR_DIMS),
    ((2, -5), (0, 1), 8, B.ERR_DIMS),
    ((2, 3), (0, 1), 2, B.ERR_ELEM_SIZE),
    ((2, 3), (0, 1), 16, B.ERR_ELEM_SIZE),
    ((1 << 16, 1 << 16), (1, 0), 4, B.ERR_TOO_LARGE),
    ((1 << 16, 1 << 15), (1, 0), 8, B.ERR_TOO_LARGE),     # 2^31 elements: element indices are 31-bit
    ((1 << 31, 1), (1, 0), 8, B.ERR_TOO_LARGE),
    ((2,) * 17, tuple(range(17)), 8, B.ERR_RANK),
    ((), (), 8, B.ERR_RANK),
])
def test_plan_create_rejects_bad_arguments(dims, perm, elem, status):
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create(dims, perm, elem)
    assert e.value.status == status


@pytest.mark.parametrize("dims,perm,elem", [
    ((1 << 15, 1 << 15), (1, 0), 8),            # 8 GiB
    ((1 << 16, 1 << 13, 2), (2, 1, 0), 4),      # 4 GiB of 4-byte elements
    ((1024, 769, 700), (2, 0, 1), 8),           # 4.4 GB, ragged
    ((16, (1 << 27) - 7), (1, 0), 4),           # nearly 2^31 elements; 16 rows half a GiB apart: the tile takes fewer
])
def test_tensors_of_4_gib_and_more_get_tile_plans(dims, perm, elem):
    """Byte offsets beyond 32 bits: the plan is flagged large and uses only the forms that exist
    for such tensors (LDS-staged tiles of 256 threads, stores first, whose positions inside a
    tile stay within the range of one buffer description)."""
    info = B.tperm_plan_create(dims, perm, elem).describe()
    assert info.large == 1 and info.volume == math.prod(dims)
    assert info.kernel_class in (B.KERNEL_TILED, B.KERNEL_PACKED)
    assert (info.threads, info.loads_first) == (256, 0)
    assert info.lds_bytes > 0 and info.nreg >= 1
    span_limit = 0xFFFFFF00
    strides_in = np.cumprod([1] + list(info.canon_dims[:info.canon_rank - 1]))
    out_dims = [info.canon_dims[info.canon_perm[j]] for j in range(info.canon_rank)]
    strides_out_by_pos = np.cumprod([1] + out_dims[:-1])
    inv = {info.canon_perm[j]: j for j in range(info.canon_rank)}
    t = info.tile_extent[:info.canon_rank]
    span_in = sum((t[z] - 1) * int(strides_in[z]) for z in range(info.canon_rank))
    span_out = sum((t[z] - 1) * int(strides_out_by_pos[inv[z]]) for z in range(info.canon_rank))
    assert (max(span_in, span_out) + 1) * info.elem_size <= span_limit


def test_large_tensor_whose_tiles_cannot_fit_falls_back_to_the_gather_kernel():
    """A 4-row matrix of 2^28 + 3 columns: any tile that holds two rows of the transposed side
    spans more than 4 GiB of the other; the gather kernel computes whole addresses."""
    info = B.tperm_plan_create(((1 << 28) + 3, 4), (1, 0), 8).describe()
    assert info.large == 1 and info.kernel_class == B.KERNEL_NAIVE
    info = B.tperm_plan_create((4, (1 << 29) - 7), (1, 0), 4).describe()
    assert info.large == 1 and info.kernel_class == B.KERNEL_NAIVE
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_forced(((1 << 28) + 3, 4), (1, 0), 8, B.KERNEL_ROWCOPY)
    assert e.value.status == B.ERR_KERNEL
    # identity permutations stay plain copies at any size
    assert B.tperm_plan_create((1 << 15, 1 << 15), (0, 1), 8).describe().kernel_class == B.KERNEL_COPY


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("dims,perm", [((70, 45, 33), (2, 0, 1)), ((301, 299), (1, 0)), ((64, 64, 64), (0, 2, 1)),
                                       ((5, 3, 7, 4, 8, 3, 9), (6, 2, 4, 0, 5, 1, 3)), ((16, 6000), (1, 0)),
                                       ((128, 128, 32), (1, 0, 2)), ((9, 7), (1, 0)), ((97, 150, 11), (1, 0, 2)),
                                       ((45, 300), (1, 0)), ((33, 257, 3), (1, 2, 0))])
def test_large_form_index_maps_on_small_tensors(dims, perm, elem):
    """large = 1 plans a small tensor the way a 4 GiB one is planned: the index maps of those
    plans, evaluated on the host with the kernel's arithmetic, against the oracle."""
    plan = _map_ok(dims, perm, elem, large=1)
    info = plan.describe()
    assert info.large == 1 and info.loads_first == 0


def test_null_arguments():
    L = B.lib()
    h = ctypes.c_void_p()
    d = (ctypes.c_int64 * 2)(2, 3)
    p = (ctypes.c_int * 2)(1, 0)
    assert L.tperm_plan_create(None, 2, d, p, 8) == B.ERR_NULL
    assert L.tperm_plan_create(ctypes.byref(h), 2, None, p, 8) == B.ERR_NULL
    assert L.tperm_plan_create(ctypes.byref(h), 2, d, None, 8) == B.ERR_NULL
    assert L.tperm_plan_destroy(None) == B.ERR_NULL
    assert L.tperm_plan_describe(None, None) == B.ERR_NULL
    assert L.tperm_execute(None, None, None, None) == B.ERR_NULL
    assert L.tperm_execute_verified(None, None, None, None, None, None, 0) == B.ERR_NULL
    assert L.tperm_multiset_compare(None, None, 4, 8, None, None, 0, None) == B.ERR_NULL
    # the checking calls validate everything on the host before anything is launched
    plan = B.tperm_plan_create((4, 5), (1, 0), 8)
    fake = ctypes.c_void_p(0x1000)
    assert L.tperm_execute_verified(plan.handle, fake, ctypes.c_void_p(0x2000), None, None, fake, 64) == B.ERR_NULL
    assert L.tperm_execute_verified(plan.handle, fake, ctypes.c_void_p(0x2000), None, ctypes.c_void_p(0x3004),
                                    ctypes.c_void_p(0x4000), 64) == B.ERR_ALIGN
    assert L.tperm_execute_verified(plan.handle, fake, ctypes.c_void_p(0x2000), None, ctypes.c_void_p(0x3000),
                                    ctypes.c_void_p(0x4000), 8) == B.ERR_TOO_LARGE
    assert L.tperm_multiset_compare(fake, fake, 4, 2, fake, fake, 64, None) == B.ERR_ELEM_SIZE
    assert L.tperm_multiset_compare(fake, fake, 0, 8, fake, fake, 64, None) == B.ERR_DIMS
    assert B.verify_workspace_bytes(1) == 64 and B.verify_workspace_bytes(16384) == 64
    assert B.verify_workspace_bytes(16385) == 128


def test_execute_without_device_reports_hip_error():
    """On a host with no GPU, execute must fail with a status, not crash or fall back."""
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    plan = B.tperm_plan_create((64, 64), (1, 0), 8)
    a = np.zeros(64 * 64, dtype=np.int64)
    b = np.zeros(64 * 64, dtype=np.int64)
    with pytest.raises(B.TpermError) as e:
        B.tperm_execute(plan, a.ctypes.data, b.ctypes.data)
    assert e.value.status == B.ERR_HIP
    assert not b.any()


@pytest.mark.parametrize("dims,perm,cdims,cperm", [
    ((2, 3, 4), (0, 1, 2), (24,), (0,)),
    ((2, 3, 4), (1, 2, 0), (2, 12), (1, 0)),
    ((2, 3, 4, 5), (2, 3, 0, 1), (6, 20), (1, 0)),
    ((2, 1, 3, 4, 1, 5), (3, 4, 5, 1, 0, 2), (6, 20), (1, 0)),
    ((1, 1, 1), (2, 0, 1), (1,), (0,)),
    ((96, 96, 96, 96), (0, 1, 3, 2), (9216, 96, 96), (0, 2, 1)),
    ((96, 96, 96, 96), (3, 0, 1, 2), (884736, 96), (1, 0)),
    ((96, 96, 96, 96), (2, 3, 0, 1), (9216, 9216), (1, 0)),
    ((96, 96, 96, 96), (3, 2, 1, 0), (96, 96, 96, 96), (3, 2, 1, 0)),
    ((5, 1, 7), (2, 1, 0), (5, 7), (1, 0)),
])
def test_canonical_form(dims, perm, cdims, cperm):
    info = B.tperm_plan_create(dims, perm, 8).describe()
    r = info.canon_rank
    assert tuple(info.canon_dims[:r]) == cdims
    assert tuple(info.canon_perm[:r]) == cperm
    assert info.volume == math.prod(dims)


def test_canonical_form_preserves_the_oracle_result():
    rng = np.random.default_rng(5)
    for _ in range(40):
        r = int(rng.integers(2, 8))
        dims = tuple(int(x) for x in rng.integers(1, 6, size=r))
        perm = tuple(int(x) for x in rng.permutation(r))
        info = B.tperm_plan_create(dims, perm, 4).describe()
        cr = info.canon_rank
        a = np.arange(math.prod(dims), dtype=np.int32)
        # a paired plan describes the same bytes as 8-byte elements
        src = a.view(np.int64) if info.paired else a
        assert info.elem_size == src.dtype.itemsize
        assert np.array_equal(oracle.transpose(a, dims, perm),
                              oracle.transpose(src, tuple(info.canon_dims[:cr]),
                                               tuple(info.canon_perm[:cr])).view(np.int32))


def test_pairing_of_four_byte_elements():
    d = lambda dims, perm, e, **kw: B.tperm_plan_create_ex(dims, perm, e, **kw).describe()
    # stride-1 dimension stays in front, even extent, 4-byte elements: paired
    info = d((6, 5, 7), (0, 2, 1), 4)
    assert info.paired == 1 and info.elem_size == 8 and info.volume == 3 * 5 * 7
    assert tuple(info.canon_dims[:info.canon_rank]) == (3, 5, 7)
    # fused leading dims count as one: (3, 4) travel together, 12 is even
    info = d((3, 4, 5, 7), (0, 1, 3, 2), 4)
    assert info.paired == 1 and tuple(info.canon_dims[:info.canon_rank]) == (6, 5, 7)
    # not paired: odd extent, leading dimension moves, 8-byte elements, copy, switched off, forced
    assert d((5, 6, 7), (0, 2, 1), 4).paired == 0
    assert d((6, 5, 7), (1, 0, 2), 4).paired == 0
    assert d((6, 5, 7), (0, 2, 1), 8).paired == 0
    assert d((6, 5, 7), (0, 1, 2), 4).paired == 0
    assert d((6, 5, 7), (0, 2, 1), 4, pair_elems=1).paired == 0
    assert d((6, 5, 7), (0, 2, 1), 4, kernel_class=B.KERNEL_PACKED).paired == 0
    assert d((6, 5, 7), (0, 2, 1), 4, kernel_class=B.KERNEL_PACKED, pair_elems=2).paired == 1
    # the map the paired plan executes is the oracle's, element by element
    rng = np.random.default_rng(11)
    for _ in range(30):
        r = int(rng.integers(2, 7))
        dims = [int(x) for x in rng.integers(1, 7, size=r)]
        dims[0] = 2 * int(rng.integers(1, 20))
        rest = rng.permutation(np.arange(1, r))
        perm = (0,) + tuple(int(x) for x in rest)
        plan = B.tperm_plan_create(dims, perm, 4)
        if not plan.describe().paired:      # canonical form was a copy
            continue
        m = B.tperm_plan_index_map(plan)
        a = np.arange(math.prod(dims), dtype=np.int32)
        assert np.array_equal(a[m], oracle.transpose(a, dims, perm))


def test_vec2_plans_move_pairs():
    """Plans that transpose even-extent leading dims move pairs of elements; the map they
    execute, evaluated on the host, is the oracle's."""
    d = lambda dims, perm, e, **kw: B.tperm_plan_create_ex(dims, perm, e, **kw).describe()
    assert d((64, 48), (1, 0), 4).vec2 == 1
    assert d((64, 48), (1, 0), 8).vec2 == 1            # 8-byte elements: 16-byte accesses
    assert d((63, 48), (1, 0), 4).vec2 == 0            # odd input leading extent
    assert d((64, 47), (1, 0), 4).vec2 == 0            # odd output leading extent
    assert d((64, 48), (1, 0), 4, vec2=1).vec2 == 0    # switched off
    assert d((64, 6, 48), (0, 2, 1), 4).vec2 == 0      # leading dim stays: paired instead
    assert d((64, 6, 48), (0, 2, 1), 4).paired == 1
    rng = np.random.default_rng(21)
    seen = 0
    for _ in range(60):
        r = int(rng.integers(2, 6))
        dims = [int(x) for x in rng.integers(1, 9, size=r)]
        perm = [int(x) for x in rng.permutation(r)]
        if perm[0] == 0:
            perm[0], perm[1] = perm[1], perm[0]
        dims[0] = 2 * int(rng.integers(1, 40))
        dims[perm[0]] = 2 * int(rng.integers(1, 40))
        elem = int(rng.choice([4, 8]))
        for kw in ({}, dict(vec2=2), dict(vec2=2, kernel_class=B.KERNEL_PACKED, m=1, tile_in=int(2 * rng.integers(1, 9)),
                                          k=1, tile_out=int(2 * rng.integers(1, 9)))):
            try:
                plan = B.tperm_plan_create_ex(dims, perm, elem, **kw)
            except B.TpermError as e:
                assert e.status == B.ERR_KERNEL
                continue
            info = plan.describe()
            seen += info.vec2
            m = B.tperm_plan_index_map(plan)
            a = np.arange(math.prod(dims), dtype=np.int32)
            assert np.array_equal(a[m], oracle.transpose(a, dims, perm)), (dims, perm, kw, B.info_dict(info))
    assert seen > 60


def test_class_selection_basics():
    k = lambda d, p, e=8: B.tperm_plan_create(d, p, e).describe().kernel_class
    assert k((1000,), (0,)) == B.KERNEL_COPY
    assert k((10, 20, 30), (0, 1, 2)) == B.KERNEL_COPY
    assert k((2048, 2048), (1, 0)) == B.KERNEL_TILED
    assert k((4, 4, 4, 4, 4, 4, 4, 4, 4), (8, 7, 6, 5, 4, 3, 2, 1, 0)) == B.KERNEL_PACKED
    assert k((4096, 64, 64), (0, 2, 1)) == B.KERNEL_ROWCOPY
    assert k((2, 64, 64, 64), (0, 2, 1, 3)) == B.KERNEL_PACKED


def test_forced_class_that_cannot_run_is_an_error():
    for kc in (B.KERNEL_TILED, B.KERNEL_COPY):
        with pytest.raises(B.TpermError) as e:
            B.tperm_plan_create_ex((8, 9, 10), (0, 2, 1), 8, kernel_class=kc)
        assert e.value.status == B.ERR_KERNEL
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_ex((8, 9, 10), (2, 1, 0), 8, kernel_class=B.KERNEL_ROWCOPY)
    assert e.value.status == B.ERR_KERNEL
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_create_ex((8, 9, 10), (0, 1, 2), 8, kernel_class=B.KERNEL_PACKED)
    assert e.value.status == B.ERR_KERNEL


# -- index maps ---------------------------------------------------------------------------

def _map_ok(dims, perm, elem, **kw):
    plan = B.tperm_plan_create_ex(dims, perm, elem, **kw)
    m = B.tperm_plan_index_map(plan)           # raises on overlap / out-of-range / LDS misuse
    vol = math.prod(dims)
    ref = oracle.transpose(np.arange(vol, dtype=np.int64), dims, perm)
    assert np.array_equal(m, ref), (dims, perm, elem, kw, B.info_dict(plan.describe()))
    return plan


def test_fig2_tile_shape():
    """The paper's tile illustration: a 9 x 7 slab cut by width-4 tiles gives 3 x 2 = 6
    tiles, two of them whole, the others ragged (Section 2.1, Figure 2)."""
    plan = _map_ok((9, 7), (1, 0), 8, kernel_class=B.KERNEL_PACKED, m=1, tile_in=4, k=1, tile_out=4)
    info = plan.describe()
    assert info.num_tiles == 6 and info.tile_volume == 16
    assert list(info.tile_extent[:2]) == [4, 4]


def test_index_maps_of_every_gpu_test_plan():
    import test_gpu_parity as G
    for elem in (8, 4):
        for dims, perm in G.SHAPES:
            _map_ok(dims, perm, elem)
            for kc in (B.KERNEL_NAIVE, B.KERNEL_TILED, B.KERNEL_PACKED, B.KERNEL_ROWCOPY):
                for ao in (1, 2):
                    try:
                        _map_ok(dims, perm, elem, kernel_class=kc, align_out=ao)
                    except B.TpermError as e:
                        assert e.status == B.ERR_KERNEL
        for dims, perm, m, tin, k, tout in G.TILES:
            for gm in (-1, 0, 1, 2, 5):
                _map_ok(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=m, tile_in=tin, k=k,
                        tile_out=tout, grid_mode=gm)


def test_line_aligned_windows_maps():
    """Aligned-window plans (halo on the read side, rows shifted to whole lines): the element
    map is the transpose, whatever the phase of the output pointer (the library evaluates the
    map at two phases and compares them itself)."""
    import test_gpu_parity as G
    for elem in (8, 4):
        for dims, perm, m, tin, k, lines in G.ALIGNED_WINDOW_TILES:
            plan = _map_ok(dims, perm, elem, m=m, tile_in=tin, k=k, tile_out=lines * (128 // elem), align_out=2)
            info = plan.describe()
            assert info.align_out == 1
            # the read side carries one line's worth of halo coordinates along the chunk
            assert info.nreg * info.threads >= math.prod(t for t in B.info_dict(info)["tile"])
    # 4-byte elements in pairs inside the windows
    for dims, perm, tin, lines in G.PAIR_WINDOW_TILES:
        info = _map_ok(dims, perm, 4, m=1, tile_in=tin, k=1, tile_out=32 * lines, align_out=2, vec2=2).describe()
        assert info.align_out == 1 and info.vec2 == 1
    # the selector takes the form by itself for misaligned low-rank transposes ...
    assert _map_ok((4001, 3777), (1, 0), 8).describe().align_out == 1
    info = _map_ok((5001, 4777), (1, 0), 4).describe()
    assert info.align_out == 1 and info.vec2 == 1
    # ... and not when rows are line-aligned or the leading output dim is short
    assert _map_ok((4096, 3072), (1, 0), 8).describe().align_out == 0
    assert _map_ok((9, 11, 13, 12, 7), (4, 3, 2, 1, 0), 8).describe().align_out == 0
    # switched off on request
    assert B.tperm_plan_create_ex((4001, 3777), (1, 0), 8, align_out=1).describe().align_out == 0


def test_index_maps_all_perms_small_grid():
    n = 0
    for dims in [(5, 4, 3), (2, 7, 3, 2), (3, 3, 3, 3), (2, 2, 3, 2, 2), (6, 1, 5, 2), (37, 11),
                 (2, 3, 2, 3, 2, 3)]:
        for perm in itertools.permutations(range(len(dims))):
            _map_ok(dims, perm, 8)
            n += 1
    assert n > 900


def test_index_maps_random_shapes_and_tiles():
    rng = np.random.default_rng(11)
    done = 0
    while done < 150:
        r = int(rng.integers(2, 9))
        dims = tuple(int(x) for x in rng.integers(1, 40, size=r))
        if math.prod(dims) > 150_000 or math.prod(dims) < 2:
            continue
        perm = tuple(int(x) for x in rng.permutation(r))
        elem = int(rng.choice([4, 8]))
        _map_ok(dims, perm, elem)
        info = B.tperm_plan_create(dims, perm, elem).describe()
        cr = info.canon_rank
        if cr >= 2:
            m = int(rng.integers(1, cr + 1))
            k = int(rng.integers(1, cr + 1))
            tin = int(rng.integers(1, info.canon_dims[m - 1] + 1))
            tout = int(rng.integers(1, info.canon_dims[info.canon_perm[k - 1]] + 1))
            try:
                _map_ok(dims, perm, elem, kernel_class=B.KERNEL_PACKED, m=m, tile_in=tin, k=k,
                        tile_out=tout, grid_mode=int(rng.integers(-1, 9)),
                        window_in=int(rng.choice([0, 1, 4, 16])), window_out=int(rng.choice([0, 1, 3, 16])),
                        threads=int(rng.choice([64, 256])), align_out=int(rng.integers(0, 3)))
            except B.TpermError as e:
                assert e.status == B.ERR_KERNEL     # tile too large for LDS / registers
        done += 1


def test_index_maps_scaled_workload_shapes():
    """The benchmark families, shrunk so the maps can be enumerated on the host."""
    for case in wl.config5()[::5]:
        dims = tuple(4 if d == 8 else 6 for d in case.dims)
        _map_ok(dims, case.perm, 4)
    for case in wl.config4()[::11]:
        scale = (300_000 / case.volume) ** (1.0 / case.rank)
        dims = tuple(max(2, int(d * scale)) for d in case.dims)
        _map_ok(dims, case.perm, 8)
    for p in itertools.permutations(range(4)):
        _map_ok((24, 20, 18, 22), p, 8)


def test_fastdiv_through_naive_descriptor():
    """The multiply-shift division is exercised on extents up to 2^31 through the naive
    kernel's map (which divides by every output extent)."""
    for dims in [(46341, 3), (3, 46337), (65536, 2), (7, 11, 13, 17), (2, 99991)]:
        perm = tuple(reversed(range(len(dims))))
        _map_ok(dims, perm, 4, kernel_class=B.KERNEL_NAIVE)


def test_selected_tiles_are_sane_for_the_benchmark_shapes():
    """Every benchmark case gets a plan; staged plans have runs of at least 128 bytes on
    both sides unless the tensor itself forbids it, and fit the LDS budget."""
    cases = wl.config1() + wl.config2() + wl.config3() + wl.config4()[::7] + wl.config5()[::4]
    for case in cases:
        info = B.tperm_plan_create(case.dims, case.perm, case.elem_size).describe()
        assert info.kernel_class in (B.KERNEL_ROWCOPY, B.KERNEL_TILED, B.KERNEL_PACKED)
        assert info.lds_bytes <= 64 * 1024
        assert info.tile_volume <= info.nreg * info.threads * (2 if info.vec2 else 1)
        # (a paired plan counts its runs in 8-byte units: info.elem_size, not the case's)
        assert info.run_out * info.elem_size >= 128, B.info_dict(info)
        if info.kernel_class != B.KERNEL_ROWCOPY:
            assert info.run_in * info.elem_size >= 128, B.info_dict(info)


def test_selector_rules_fitted_to_measurements():
    """The measured rules of the selector, pinned on the shapes they came from."""
    d = lambda dims, perm, e, **kw: B.info_dict(B.tperm_plan_create_ex(dims, perm, e, **kw).describe())
    # rows a multiple of 8 KiB apart: at most 32 of them per tile (96^4, permutations 2013 and 3012)
    for perm in ((2, 0, 1, 3), (3, 0, 1, 2)):
        info = d((96, 96, 96, 96), perm, 8)
        rows = math.prod(info["tile"][1:])
        assert info["kernel"] == "tiled" and rows <= 32, info
    # ... while rows 768 bytes apart may be many (permutation 1023)
    assert math.prod(d((96, 96, 96, 96), (1, 0, 2, 3), 8)["tile"][1:]) >= 64
    # the LDS-free row copy takes four to six slots per thread when they come from several rows
    info = d((96, 96, 96, 96), (0, 2, 3, 1), 8)
    assert info["kernel"] == "rowcopy" and info["nreg"] in (4, 6), info
    # 4-byte elements: windows with pairs for misaligned rows, not when the input rows are line-aligned
    assert d((13953, 13953), (1, 0), 4)["align_out"] == 1 and d((13953, 13953), (1, 0), 4)["vec2"] == 1
    assert d((6560, 6103), (1, 0), 4)["align_out"] == 0
    assert d((6560, 6103), (1, 0), 4)["cache_policy"] == 4     # nontemporal loads only
    # a short leading output dim needs one window chunk more out of a few: plain tiles there
    assert d((224, 367, 191), (2, 1, 0), 8)["align_out"] == 0
    assert d((12688, 11907), (1, 0), 8)["align_out"] == 1


def test_planner_under_address_and_ub_sanitizers(tmp_path):
    """The planner (pure host C++) is built with ASan + UBSan and driven with random problems
    and options; every plan's index map must be a bijection and no sanitizer may fire."""
    import shutil
    import subprocess
    if shutil.which("g++") is None:
        pytest.skip("g++ not available")
    exe = str(tmp_path / "planner_fuzz")
    src = [os.path.join(ROOT, "tests", "planner_fuzz.cpp"),
           os.path.join(ROOT, "paper_1705_01598_amd", "csrc", "plan.cpp"),
           os.path.join(ROOT, "paper_1705_01598_amd", "csrc", "model.cpp")]
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-I" + os.path.join(ROOT, "include"),
                    *src, "-o", exe], check=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=1"
    r = subprocess.run([exe, "1500"], capture_output=True, text=True, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok:"), r.stdout + r.stderr


def _transpose_status(dims, perm, elem, a=None, b=None):
    rank = len(dims)
    cd = (ctypes.c_int64 * max(rank, 1))(*dims)
    cp = (ctypes.c_int * max(rank, 1))(*perm)
    pa = a.ctypes.data if a is not None else None
    pb = b.ctypes.data if b is not None else None
    return B.lib().tperm_transpose(rank, cd, cp, elem, pa, pb, None)


def test_plan_cache_on_the_host():
    """The cache keeps one plan per problem, counts hits and misses, evicts beyond its
    capacity and reports plan-creation errors unchanged.  (Without a GPU the execute step of
    tperm_transpose fails with the HIP status after the plan has been cached.)"""
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: covered by the GPU tests")
    B.tperm_cache_clear()
    assert B.tperm_cache_stats() == {"entries": 0, "hits": 0, "misses": 0}
    a = np.zeros(6 * 5 * 7, dtype=np.int64)
    b = np.zeros_like(a)
    assert _transpose_status((6, 5, 7), (2, 0, 1), 8, a, b) == B.ERR_HIP
    assert B.tperm_cache_stats() == {"entries": 1, "hits": 0, "misses": 1}
    assert _transpose_status((6, 5, 7), (2, 0, 1), 8, a, b) == B.ERR_HIP
    assert B.tperm_cache_stats() == {"entries": 1, "hits": 1, "misses": 1}
    # same extents, other permutation or element size: other entries
    assert _transpose_status((6, 5, 7), (1, 0, 2), 8, a, b) == B.ERR_HIP
    assert _transpose_status((6, 5, 7), (2, 0, 1), 4, a, b) == B.ERR_HIP
    assert B.tperm_cache_stats()["entries"] == 3
    # argument errors come back as they would from plan creation / execute; nothing is cached
    assert _transpose_status((6, 5, 7), (2, 0, 0), 8, a, b) == B.ERR_PERM
    assert _transpose_status((6, 0, 7), (2, 0, 1), 8, a, b) == B.ERR_DIMS
    assert _transpose_status((6, 5, 7), (2, 0, 1), 2, a, b) == B.ERR_ELEM_SIZE
    assert _transpose_status((), (), 8, a, b) == B.ERR_RANK
    assert _transpose_status((6, 5, 7), (2, 0, 1), 8, a, a) == B.ERR_ALIAS
    assert _transpose_status((6, 5, 7), (2, 0, 1), 8, None, b) == B.ERR_NULL
    assert B.lib().tperm_transpose(3, None, None, 8, None, None, None) == B.ERR_NULL
    assert B.tperm_cache_stats()["entries"] == 3
    # capacity: least recently used entries go first
    for n in range(2, 4200):
        _transpose_status((n, 3), (1, 0), 8, a, b)
    s = B.tperm_cache_stats()
    assert s["entries"] == 4096
    hits = s["hits"]
    _transpose_status((4199, 3), (1, 0), 8, a, b)      # recent: still there
    assert B.tperm_cache_stats()["hits"] == hits + 1
    _transpose_status((6, 5, 7), (2, 0, 1), 8, a, b)   # oldest: evicted, so a miss
    assert B.tperm_cache_stats()["hits"] == hits + 1
    B.tperm_cache_clear()
    assert B.tperm_cache_stats() == {"entries": 0, "hits": 0, "misses": 0}


def test_plan_cache_is_thread_safe():
    torch = pytest.importorskip("torch")
    if torch.cuda.is_available():
        pytest.skip("a GPU is present: covered by the GPU tests")
    import threading
    B.tperm_cache_clear()
    a = np.zeros(64, dtype=np.int64)
    b = np.zeros_like(a)
    errors = []

    def worker(seed):
        rng = np.random.default_rng(seed)
        for i in range(300):
            n = int(rng.integers(2, 40))
            if _transpose_status((n, 3, 2), (2, 0, 1), 8, a, b) != B.ERR_HIP:
                errors.append((seed, i))
            if i % 97 == 0:
                B.tperm_cache_clear()

    ts = [threading.Thread(target=worker, args=(s,)) for s in range(8)]
    for t in ts:
        t.start()
    for t in ts:
        t.join()
    assert not errors
    assert B.tperm_cache_stats()["entries"] <= 38
    B.tperm_cache_clear()


# -- analytical model (Section 2.3, Eqs. (10)-(13)) --------------------------------------------
def _lines_of(byte_ranges):
    """Distinct 128-byte lines of a list of (begin, nbytes), and how many receive all 128 bytes."""
    got = {}
    for b0, nb in byte_ranges:
        for byte in range(b0, b0 + nb):
            got[byte // 128] = got.get(byte // 128, 0) + 1
    return len(got), sum(1 for v in got.values() if v == 128)


@pytest.mark.parametrize("d0,d1,t0,t1", [(40, 24, 20, 12), (33, 50, 33, 25), (64, 64, 32, 32), (35, 18, 16, 9)])
def test_model_line_counts_against_enumeration(d0, d1, t0, t1):
    """2-D transposes cut into at most 8 tiles: the model walks every tile, so its averages
    must equal a direct enumeration of the bytes each tile reads and writes."""
    plan = B.tperm_plan_create_ex((d0, d1), (1, 0), 8, kernel_class=B.KERNEL_PACKED, m=1, tile_in=t0, k=1,
                                  tile_out=t1, vec2=1, align_out=1)
    info = plan.describe()
    assert list(info.tile_extent[:2]) == [t0, t1] and info.num_tiles <= 8
    m = B.tperm_plan_model(plan)
    ld = st = full = tiles = 0
    for a0 in range(0, d0, t0):
        for a1 in range(0, d1, t1):
            i0 = range(a0, min(a0 + t0, d0))
            i1 = range(a1, min(a1 + t1, d1))
            n, _ = _lines_of([((x + d0 * y) * 8, 8) for x in i0 for y in i1])       # input: dims[0] fastest
            ld += n
            n, f = _lines_of([((y + d1 * x) * 8, 8) for x in i0 for y in i1])       # output: input dim 1 fastest
            st += n
            full += f
            tiles += 1
    assert tiles == info.num_tiles
    assert m.ld_tran == pytest.approx(ld / tiles) and m.st_tran == pytest.approx(st / tiles)
    assert m.cl_full == pytest.approx(full / tiles) and m.cl_part == pytest.approx((st - full) / tiles)
    assert m.useful_bytes_per_tile == pytest.approx(d0 * d1 * 8 / tiles)
    assert m.ld_req == info.nreg * info.threads / 64 and m.mlp == info.nreg
    # Eq. (13) from the counted quantities
    part = m.cl_part / max(1.0, m.cl_full + m.cl_part)
    assert m.tpr_mem == pytest.approx((m.ld_tran + m.st_tran * (1 + part)) / (m.ld_req + m.st_req))
    assert 1 <= m.ld_runs <= m.ld_tran and 1 <= m.st_runs <= m.st_tran
    assert m.cycles_total == pytest.approx((m.cycles_mem + m.cycles_lds + m.cycles_ac) * m.n_iter)   # Eq. (10)


def test_model_sampled_line_counts_track_the_whole_tensor():
    """More tiles than the model samples: line-aligned tiles have a closed form, and on a ragged
    matrix the sampled estimate stays close to an enumeration of every tile (the ragged edge
    tiles, which a sample can over- or under-represent, must not shift the totals)."""
    tile = dict(kernel_class=B.KERNEL_PACKED, m=1, k=1, vec2=1, align_out=1)
    m = B.tperm_plan_model(B.tperm_plan_create_ex((4096, 4096), (1, 0), 8, tile_in=32, tile_out=32, **tile))
    assert (m.ld_tran, m.st_tran, m.cl_full, m.cl_part) == (64, 64, 64, 0)     # 32 rows of 256 bytes either way
    assert m.useful_bytes_per_tile == 32 * 32 * 8
    d0, d1, t = 301, 299, 32
    plan = B.tperm_plan_create_ex((d0, d1), (1, 0), 8, tile_in=t, tile_out=t, **tile)
    info = plan.describe()
    m = B.tperm_plan_model(plan)
    ld = st = full = tiles = 0
    for a0 in range(0, d0, t):
        for a1 in range(0, d1, t):
            i0 = range(a0, min(a0 + t, d0))
            i1 = range(a1, min(a1 + t, d1))
            n, _ = _lines_of([((x + d0 * y) * 8, 8) for x in i0 for y in i1])
            ld += n
            n, f = _lines_of([((y + d1 * x) * 8, 8) for x in i0 for y in i1])
            st += n
            full += f
            tiles += 1
    assert tiles == info.num_tiles == 100
    assert m.useful_bytes_per_tile == pytest.approx(d0 * d1 * 8 / tiles)
    assert m.ld_tran == pytest.approx(ld / tiles, rel=0.05) and m.st_tran == pytest.approx(st / tiles, rel=0.05)
    assert m.cl_part == pytest.approx((st - full) / tiles, rel=0.10)


def test_model_prices_partial_lines_and_short_runs():
    us = lambda dims, perm, **kw: B.tperm_plan_model(B.tperm_plan_create_ex(dims, perm, 8, **kw)).microseconds
    tile = dict(kernel_class=B.KERNEL_PACKED, m=1, k=1, vec2=1, align_out=1)
    # rows that start anywhere in a line cost more than line-aligned ones of nearly the same size
    assert us((4097, 4097), (1, 0), tile_in=32, tile_out=32, **tile) > 1.2 * us((4096, 4096), (1, 0), tile_in=32, tile_out=32, **tile)
    # 4-element output pieces (partial lines everywhere) against 32-element ones
    assert us((4096, 4096), (1, 0), tile_in=256, tile_out=4, **tile) > 1.5 * us((4096, 4096), (1, 0), tile_in=32, tile_out=32, **tile)
    with pytest.raises(B.TpermError) as e:
        B.tperm_plan_model(B.tperm_plan_create((5, 6, 7), (0, 1, 2), 8))           # a plain copy has no tile
    assert e.value.status == B.ERR_KERNEL


def test_model_selector_builds_valid_plans():
    """Plans chosen by the analytical model (selector = 1) still map every element correctly."""
    rng = np.random.default_rng(31)
    for dims, perm, elem in [((70, 45, 33, 6), (2, 0, 3, 1), 8), ((8, 8, 8, 8, 8), (1, 3, 0, 2, 4), 4),
                             ((129, 7, 65), (2, 1, 0), 8), ((33, 5, 7, 16, 3), (0, 3, 1, 4, 2), 4), ((301, 299), (1, 0), 8)]:
        plan = _map_ok(dims, perm, elem, selector=1)
        assert plan.describe().kernel_class in (B.KERNEL_ROWCOPY, B.KERNEL_TILED, B.KERNEL_PACKED)
