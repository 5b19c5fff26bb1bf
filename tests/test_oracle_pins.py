"""Pins for the CPU oracle: it is checked against what the paper's definition and plain
mathematics fix, never against itself or the GPU path.

Each pin is chosen so that a plausible slip (gather/scatter direction swapped, a stride
taken from the wrong layout, a transposed operand, a dropped dimension) fails it.
"""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _u(a):
    """Raw-bit view for bit-exact comparison."""
    a = np.ascontiguousarray(a)
    return a.view({4: np.uint32, 8: np.uint64}[a.dtype.itemsize])


def _rand(vol, elem, seed):
    rng = np.random.default_rng(seed)
    dt = np.uint64 if elem == 8 else np.uint32
    return rng.integers(0, np.iinfo(dt).max, size=vol, dtype=dt)


FORMS_C = [oracle.transpose, oracle.transpose_scatter]


# -- 1. identity permutation is a copy (the trivial permutation of Section 3.2) ---------
@pytest.mark.parametrize("form", FORMS_C + [oracle.transpose_numpy])
@pytest.mark.parametrize("dims", [(7,), (5, 3), (2, 3, 4), (3, 1, 4, 2), (2, 2, 2, 2, 3)])
def test_identity_is_copy(form, dims):
    a = _rand(math.prod(dims), 8, 1)
    assert np.array_equal(form(a, dims, tuple(range(len(dims)))), a)


# -- 2. rank 2, perm (1,0) is the matrix transpose: closed form written out -------------
@pytest.mark.parametrize("form", FORMS_C)
@pytest.mark.parametrize("d0,d1", [(1, 1), (1, 5), (5, 1), (3, 4), (9, 7), (33, 65)])
def test_rank2_closed_form(form, d0, d1):
    a = _rand(d0 * d1, 4, 2)
    b = form(a, (d0, d1), (1, 0))
    for i in range(d0):
        for j in range(d1):
            assert b[j + i * d1] == a[i + j * d0]


# -- 3. rank-3 cyclic permutation: tells the gather reading from the scatter reading ----
@pytest.mark.parametrize("form", FORMS_C + [oracle.transpose_numpy])
def test_rank3_cyclic_direction(form):
    dims, perm = (2, 3, 4), (1, 2, 0)
    assert oracle.out_dims(dims, perm) == [3, 4, 2]
    a = np.arange(24, dtype=np.int64)
    b = form(a, dims, perm)
    for y0, y1, y2 in itertools.product(range(2), range(3), range(4)):
        assert b[y1 + 3 * y2 + 12 * y0] == a[y0 + 2 * y1 + 6 * y2]
    # the opposite (scatter-direction) reading would give extents (4, 2, 3) and
    # B[y2 + 4*y0 + 8*y1]; make sure that is NOT what comes out
    wrong = np.empty_like(a)
    for y0, y1, y2 in itertools.product(range(2), range(3), range(4)):
        wrong[y2 + 4 * y0 + 8 * y1] = a[y0 + 2 * y1 + 6 * y2]
    assert not np.array_equal(b, wrong)


# -- 3b. the paper's printed Eq. (1), taken literally, is only right for involutions ----
def test_eq1_literal_reading_differs_for_non_involution():
    dims, perm = (2, 3, 4), (1, 2, 0)
    r = 3
    sI = [math.prod(dims[:z]) for z in range(r)]
    sO = [math.prod([dims[perm[t]] for t in range(j)]) for j in range(r)]
    a = np.arange(24, dtype=np.int64)
    literal = np.full(24, -1, dtype=np.int64)
    for p in range(24):
        # coordinate of input dim i times the output stride of the dim at position i
        q = sum(((p // sI[i]) % dims[i]) * sO[i] for i in range(r))
        literal[q % 24] = a[p]
    assert not np.array_equal(literal, oracle.transpose_scatter(a, dims, perm))


# -- 4. brute force over every permutation of a grid of tiny shapes ---------------------
def _tiny_shapes():
    shapes = []
    for r in range(1, 5):
        for dims in itertools.product((1, 2, 3, 5), repeat=r):
            if math.prod(dims) <= 60:
                shapes.append(dims)
    shapes += [(2, 3, 2, 2, 3), (1, 2, 1, 3, 2), (4, 3, 2, 1, 2), (2, 2, 2, 2, 2, 2)]
    return shapes


def test_bruteforce_all_perms_tiny():
    n = 0
    for dims in _tiny_shapes():
        vol = math.prod(dims)
        a = np.arange(vol, dtype=np.int32) * 7 + 3
        for perm in itertools.permutations(range(len(dims))):
            ref = np.array(oracle.transpose_bruteforce(a.tolist(), dims, perm), dtype=np.int32)
            assert np.array_equal(oracle.transpose(a, dims, perm), ref), (dims, perm)
            assert np.array_equal(oracle.transpose_scatter(a, dims, perm), ref), (dims, perm)
            assert np.array_equal(oracle.transpose_numpy(a, dims, perm), ref), (dims, perm)
            n += 1
    assert n > 3000


# -- 5. inverse permutation restores the input; composition law -------------------------
@pytest.mark.parametrize("seed", range(12))
def test_inverse_and_composition(seed):
    rng = np.random.default_rng(100 + seed)
    r = int(rng.integers(2, 8))
    dims = tuple(int(x) for x in rng.integers(1, 7, size=r))
    p = tuple(int(x) for x in rng.permutation(r))
    q = tuple(int(x) for x in rng.permutation(r))
    a = _rand(math.prod(dims), 8, seed)
    tp = oracle.transpose(a, dims, p)
    od = oracle.out_dims(dims, p)
    # T_inv(p) T_p = identity
    assert np.array_equal(oracle.transpose(tp, od, oracle.inverse_perm(p)), a)
    # T_q T_p = T_{p o q} with (p o q)[j] = p[q[j]]  (follows from the gather convention)
    pq = tuple(p[q[j]] for j in range(r))
    assert np.array_equal(oracle.transpose(tp, od, q), oracle.transpose(a, dims, pq))


# -- 6. index stamp: the output is a permutation of the input's multiset, and the stamp
#       found at output position o is the input position the definition assigns to it ----
@pytest.mark.parametrize("seed", range(8))
def test_stamp_multiset_and_positions(seed):
    rng = np.random.default_rng(200 + seed)
    r = int(rng.integers(2, 7))
    dims = tuple(int(x) for x in rng.integers(2, 9, size=r))
    perm = tuple(int(x) for x in rng.permutation(r))
    vol = math.prod(dims)
    a = np.arange(vol, dtype=np.int64)
    b = oracle.transpose(a, dims, perm)
    assert np.array_equal(np.sort(b), a)
    sI = [math.prod(dims[:z]) for z in range(r)]
    for o in rng.integers(0, vol, size=50):
        x = []
        rem = int(o)
        for j in range(r):
            x.append(rem % dims[perm[j]])
            rem //= dims[perm[j]]
        expect = sum(x[j] * sI[perm[j]] for j in range(r))
        assert b[o] == expect
        assert oracle.input_position(dims, perm, int(o)) == expect
    pos = rng.integers(0, vol, size=64)
    assert np.array_equal(oracle.sample(a, dims, perm, pos), b[pos])


# -- 7. library special case on medium random shapes, both element sizes, all C forms ---
@pytest.mark.parametrize("elem", [4, 8])
@pytest.mark.parametrize("seed", range(10))
def test_numpy_library_form_medium(seed, elem):
    rng = np.random.default_rng(300 + seed)
    r = int(rng.integers(2, 9))
    dims = tuple(int(x) for x in rng.integers(1, 10, size=r))
    while math.prod(dims) > 300_000:
        dims = dims[:-1]
    perm = tuple(int(x) for x in rng.permutation(len(dims)))
    a = _rand(math.prod(dims), elem, seed)
    ref = oracle.transpose_numpy(a, dims, perm)
    assert np.array_equal(oracle.transpose(a, dims, perm), ref)
    assert np.array_equal(oracle.transpose_scatter(a, dims, perm), ref)
    assert np.array_equal(oracle.transpose(a, dims, perm, nthreads=1), ref)
    assert np.array_equal(oracle.transpose(a, dims, perm, nthreads=3), ref)


# -- 8. config 1 at full size against the library form ----------------------------------
def test_config1_full_size_vs_numpy():
    case = wl.config1()[0]
    a = wl.uniform_values(case)
    assert a.dtype == np.float64 and a.min() >= -1.0 and a.max() < 1.0
    b = oracle.transpose(a, case.dims, case.perm)
    m = a.reshape(2048, 2048)          # C order: m[j, i] = a[i + 2048 j]
    assert np.array_equal(_u(b), _u(np.ascontiguousarray(m.T).reshape(-1)))


# -- 9. raw bits survive: NaN payloads, -0.0, denormals, infinities ---------------------
@pytest.mark.parametrize("elem", [4, 8])
def test_bits_survive(elem):
    case = wl.make_case(0, 1, (5, 4, 3), (2, 0, 1), elem)
    a = wl.bitpattern_values(case)
    fl = a.view(np.float64 if elem == 8 else np.float32)
    b = oracle.transpose(fl, case.dims, case.perm)
    assert np.array_equal(np.sort(_u(b)), np.sort(a))
    assert np.array_equal(_u(b), oracle.transpose_numpy(a, case.dims, case.perm))


# -- 10. extent-1 dimensions and dimension fusing leave the result unchanged -------------
def test_unit_extents_and_fusing_preserve_result():
    a = _rand(2 * 3 * 4 * 5, 8, 5)
    # (2,3,4,5) perm (2,3,0,1): dims {0,1} and {2,3} travel together -> (6,20) perm (1,0)
    assert np.array_equal(oracle.transpose(a, (2, 3, 4, 5), (2, 3, 0, 1)),
                          oracle.transpose(a, (6, 20), (1, 0)))
    # inserting extent-1 dimensions anywhere changes nothing
    assert np.array_equal(oracle.transpose(a, (2, 1, 3, 4, 1, 5), (3, 4, 5, 1, 0, 2)),
                          oracle.transpose(a, (6, 20), (1, 0)))


# -- 11. argument checking ----------------------------------------------------------------
def test_rejects_bad_arguments():
    a = np.zeros(6, dtype=np.int32)
    with pytest.raises(ValueError):
        oracle.transpose(a, (2, 3), (0, 0))
    with pytest.raises(ValueError):
        oracle.transpose(a, (2, 3), (0, 2))
    with pytest.raises(ValueError):
        oracle.transpose(a, (2, 0), (0, 1))
    with pytest.raises(ValueError):
        oracle.transpose(a, (2, 4), (1, 0))


# -- 12. shapes the paper prints (Section 3.2): volumes pin the extracted extents --------
def test_golden_set2_shapes():
    rows = {}
    with open(os.path.join(GOLDEN, "set2_shapes.txt")) as fh:
        for line in fh:
            line = line.split("#")[0].strip()
            if line:
                name, dims, approx = line.split(";")
                rows[name.strip()] = (tuple(int(x) for x in dims.split(",")), float(approx))
    assert rows["rank8"][0] == wl.SET2_RANK8_DIMS
    assert rows["rank12"][0] == wl.SET2_RANK12_DIMS
    for dims, approx_millions in rows.values():
        assert abs(math.prod(dims) / 1e6 - approx_millions) < 6.0
    # reverse permutation of the rank-8 shape, scaled down by keeping the small extents:
    dims = (5, 3, 2, 4, 3, 3, 2, 2)
    rev = tuple(reversed(range(8)))
    a = _rand(math.prod(dims), 8, 9)
    assert np.array_equal(oracle.transpose(a, dims, rev),
                          np.ascontiguousarray(a.reshape(dims, order="F").reshape(-1, order="C")))


# -- 13. accumulate mode (Section 3.3): out + transposed in, one IEEE addition per element ---
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_accumulate_form(dtype):
    rng = np.random.default_rng(77)
    for _ in range(10):
        r = int(rng.integers(1, 6))
        dims = tuple(int(x) for x in rng.integers(1, 8, size=r))
        perm = tuple(int(x) for x in rng.permutation(r))
        vol = math.prod(dims)
        a = rng.standard_normal(vol).astype(dtype)
        b = rng.standard_normal(vol).astype(dtype)
        got = oracle.transpose_accumulate(a, b, dims, perm)
        # library form: the addition is elementwise on the transposed input, same dtype
        ref = b + oracle.transpose_numpy(a, dims, perm)
        assert got.dtype == dtype and np.array_equal(_u(got), _u(ref))
        # onto zeros it is the plain transpose (x + 0 keeps every finite x, -0.0 aside)
        z = oracle.transpose_accumulate(a, np.zeros(vol, dtype=dtype), dims, perm)
        assert np.array_equal(z, oracle.transpose(a, dims, perm))
    # small integers are exact: accumulating twice doubles
    a = np.arange(24, dtype=dtype)
    once = oracle.transpose_accumulate(a, np.zeros(24, dtype=dtype), (2, 3, 4), (2, 0, 1))
    twice = oracle.transpose_accumulate(a, once, (2, 3, 4), (2, 0, 1))
    assert np.array_equal(twice, 2 * once)


# -- 14. contraction D + L * R as a direct loop nest (Section 3.4) ----------------------------
def test_contract_hand_computed_2x2x2():
    """D[a,b] += sum_k L[a,k] R[k,b] with a, b, k of extent 2, worked by hand.  Flat buffers,
    first label fastest: L = [L00, L10, L01, L11] = [1, 2, 3, 4], R = [R00, R10, R01, R11] =
    [5, 6, 7, 8], D starts as [10, 20, 30, 40]."""
    l = np.array([1.0, 2.0, 3.0, 4.0])
    r = np.array([5.0, 6.0, 7.0, 8.0])
    d = np.array([10.0, 20.0, 30.0, 40.0])
    # D00 = 10 + 1*5 + 3*6 = 33   D10 = 20 + 2*5 + 4*6 = 54
    # D01 = 30 + 1*7 + 3*8 = 61   D11 = 40 + 2*7 + 4*8 = 86
    got = oracle.contract("ab", "ak", "kb", dict(a=2, b=2, k=2), l, r, d)
    assert got.tolist() == [33.0, 54.0, 61.0, 86.0]
    assert d.tolist() == [10.0, 20.0, 30.0, 40.0]            # the destination passed in is untouched
    # the result stored transposed ("ba"): D[b,a], b fastest, starting from the same numbers
    got_t = oracle.contract("ba", "ak", "kb", dict(a=2, b=2, k=2), l, r, np.array([10.0, 30.0, 20.0, 40.0]))
    assert got_t.tolist() == [33.0, 61.0, 54.0, 86.0]
    # an operand stored transposed ("ka": k fastest) holding the same matrix
    got_l = oracle.contract("ab", "ka", "kb", dict(a=2, b=2, k=2), np.array([1.0, 3.0, 2.0, 4.0]), r, d)
    assert got_l.tolist() == [33.0, 54.0, 61.0, 86.0]


@pytest.mark.parametrize("dtype", [np.float64, np.float32])
def test_contract_is_the_matrix_product(dtype):
    """One free label each and one summed label: the closed form is the matrix product; with
    small integers every product and sum is exact, so the comparison is bit for bit."""
    rng = np.random.default_rng(11)
    for a, b, k in [(3, 5, 4), (1, 7, 2), (6, 1, 5), (4, 4, 1)]:
        L = rng.integers(-4, 5, size=(a, k)).astype(dtype)
        R = rng.integers(-4, 5, size=(k, b)).astype(dtype)
        D = rng.integers(-9, 10, size=(a, b)).astype(dtype)
        got = oracle.contract("ab", "ak", "kb", dict(a=a, b=b, k=k), L.ravel(order="F"), R.ravel(order="F"),
                              D.ravel(order="F"))
        assert got.dtype == dtype and np.array_equal(got, (D + L @ R).ravel(order="F"))


def test_contract_matches_nested_python_loops():
    """Several labels on every side, all tensors in scrambled layouts: pure-Python loops over
    every combination of label values."""
    ext = dict(a=2, b=3, c=2, d=3, e=2)
    d_lab, l_lab, r_lab = "bea", "dacb", "ced"            # summed: d, c; free: a, b from L; e from R
    rng = np.random.default_rng(12)
    vol = lambda s: math.prod(ext[c] for c in s)
    l = rng.integers(-3, 4, size=vol(l_lab)).astype(np.float64)
    r = rng.integers(-3, 4, size=vol(r_lab)).astype(np.float64)
    d = rng.integers(-3, 4, size=vol(d_lab)).astype(np.float64)

    def pos(labels, val):
        p, stride = 0, 1
        for c in labels:
            p += val[c] * stride
            stride *= ext[c]
        return p

    want = d.copy()
    names = sorted(ext)
    for combo in itertools.product(*[range(ext[c]) for c in names]):
        val = dict(zip(names, combo))
        want[pos(d_lab, val)] += l[pos(l_lab, val)] * r[pos(r_lab, val)]
    assert np.array_equal(oracle.contract(d_lab, l_lab, r_lab, ext, l, r, d), want)


def test_contract_commutes_with_the_transpose_oracle():
    """Storing an operand in another layout (the gather transpose of it) and relabelling
    accordingly leaves the result unchanged; storing the result in another layout transposes
    it.  Ties the contraction's layout convention to the transpose's."""
    ext = dict(a=3, b=2, c=4, k=3, j=2)
    rng = np.random.default_rng(13)
    vol = lambda s: math.prod(ext[c] for c in s)
    dims = lambda s: tuple(ext[c] for c in s)
    l_lab, r_lab, d_lab = "akbj", "jck", "abc"
    # small integers: every sum is exact whatever the order of the summed labels
    l = rng.integers(-5, 6, size=vol(l_lab)).astype(np.float64)
    r = rng.integers(-5, 6, size=vol(r_lab)).astype(np.float64)
    d = rng.integers(-5, 6, size=vol(d_lab)).astype(np.float64)
    base = oracle.contract(d_lab, l_lab, r_lab, ext, l, r, d)
    l2_lab = "jbka"
    l2 = oracle.transpose(l, dims(l_lab), tuple(l_lab.index(c) for c in l2_lab))
    assert np.array_equal(oracle.contract(d_lab, l2_lab, r_lab, ext, l2, r, d), base)
    d2_lab = "cab"
    perm = tuple(d_lab.index(c) for c in d2_lab)
    d2 = oracle.transpose(d, dims(d_lab), perm)
    assert np.array_equal(oracle.contract(d2_lab, l_lab, r_lab, ext, l, r, d2), oracle.transpose(base, dims(d_lab), perm))
    for bad in [("ab", "ak", "kk"), ("ab", "ak", "jb"), ("abk", "ak", "kb"), ("ab", "akc", "kb")]:
        with pytest.raises(ValueError):
            oracle.contract(*bad, dict(a=2, b=2, c=2, j=2, k=2), np.zeros(8), np.zeros(8), np.zeros(8))
