"""Tensor contraction through transposes + GEMM (application layer on top of the library).

The checker is the oracle's direct loop nest (oracle.contract: one output element at a time,
products summed in double precision in a fixed order; pinned in test_oracle_pins.py on a
hand-computed case, the matrix product, nested Python loops and the transpose oracle).
CPU part: the label bookkeeping is checked by emulating the four steps with the oracle's
transposes and numpy's matrix product.  GPU part: the real path (tperm transposes, vendor GEMM
through torch.mm, accumulating transpose) against the oracle; a GEMM sums in another order
than the loop nest, so this comparison has a tolerance, unlike every transpose test: with K
products per output element, each rounded in the working precision (unit roundoff eps), the
error of either summation order is at most about K * eps * sum_k |l||r| (the standard bound
for recursive summation), so |difference| <= 2 * 8 * K * eps * sum_k |l||r| + 8 * eps * |ref|
per output element (factor 8: slack for fused multiply-adds and blocked partial sums)."""
import math

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import contraction as C
from paper_1705_01598_amd import workloads as wl

SMALL = [
    ("ab", "ak", "kb", dict(a=5, b=7, k=3)),                       # plain matrix product
    ("ba", "ak", "kb", dict(a=5, b=7, k=3)),                       # transposed result
    ("abef", "abcd", "cdef", dict(a=3, b=4, c=2, d=5, e=3, f=2)),  # no transposes needed
    ("ebfa", "cadb", "fdce", dict(a=3, b=4, c=2, d=5, e=3, f=2)),  # all four steps permute
    ("cab", "bkc", "ak", dict(a=4, b=3, c=5, k=6)),
]


def _oracle_ref(lay, l, r, d):
    """d + l * r by the oracle's loop nest (first label = stride-1 dimension)."""
    return oracle.contract(lay.d_labels, lay.l_labels, lay.r_labels, dict(lay.extents), l, r, d)


@pytest.mark.parametrize("d,l,r,ext", SMALL)
def test_layout_bookkeeping_reproduces_the_oracle(d, l, r, ext):
    lay = C.layout(d, l, r, ext)
    rng = np.random.default_rng(3)
    lv = rng.standard_normal(math.prod(lay.dims(l)))
    rv = rng.standard_normal(math.prod(lay.dims(r)))
    dv = rng.standard_normal(math.prod(lay.dims(d)))
    lp = oracle.transpose(lv, lay.dims(l), lay.l_perm)                 # (free_l, summed): m x k
    rp = oracle.transpose(rv, lay.dims(r), lay.r_perm)                 # (summed, free_r): k x n
    t = (lp.reshape((lay.m, lay.k), order="F") @ rp.reshape((lay.k, lay.n), order="F")).ravel(order="F")
    got = oracle.transpose_accumulate(t, dv, lay.dims(lay.free_l + lay.free_r), lay.t_perm)
    assert np.allclose(got, _oracle_ref(lay, lv, rv, dv), rtol=1e-12, atol=1e-12)
    assert lay.flops == 2 * lay.m * lay.n * lay.k


def test_layout_rejects_bad_specifications():
    for d, l, r in [("ab", "ak", "kk"), ("ab", "ak", "jb"), ("abk", "ak", "kb"), ("ab", "akc", "kb"), ("ab", "ab", "ab")]:
        with pytest.raises(ValueError):
            C.layout(d, l, r, dict(a=2, b=2, c=2, j=2, k=2))
    with pytest.raises(ValueError):
        C.layout("ab", "ak", "kb", dict(a=2, b=2))


def test_arithmetic_intensity_formula():
    lay = C.layout("ab", "ak", "kb", dict(a=100, b=100, k=100))
    assert lay.arithmetic_intensity == pytest.approx(2 * math.sqrt(1e12) / 3e4)
    for case in wl.contraction_cases():
        lay = C.layout(case["d"], case["l"], case["r"], case["extents"])
        assert max(len(case["d"]), len(case["l"]), len(case["r"])) <= 8
        assert max(lay.m * lay.n, lay.m * lay.k, lay.k * lay.n) < 1 << 26


@pytest.mark.gpu
@pytest.mark.parametrize("dtype_name", ["float64", "float32"])
@pytest.mark.parametrize("d,l,r,ext", SMALL + [
    ("ebfa", "cadb", "fdce", dict(a=30, b=14, c=12, d=9, e=20, f=16)),
    ("dabfec", "aghcbi", "efdghi", dict(a=4, b=6, c=5, d=3, e=4, f=3, g=7, h=2, i=5)),
])
def test_gpu_contraction_matches_the_oracle(d, l, r, ext, dtype_name):
    torch = pytest.importorskip("torch")
    dtype = getattr(torch, dtype_name)
    lay = C.layout(d, l, r, ext)
    rng = np.random.default_rng(5)
    npdt = np.float64 if dtype == torch.float64 else np.float32
    lv = (rng.random(math.prod(lay.dims(l))) * 2 - 1).astype(npdt)
    rv = (rng.random(math.prod(lay.dims(r))) * 2 - 1).astype(npdt)
    dv = (rng.random(math.prod(lay.dims(d))) * 2 - 1).astype(npdt)
    d_dev = torch.from_numpy(dv.copy()).cuda()
    con = C.Contraction(d, l, r, ext, dtype)
    con.run(torch.from_numpy(lv).cuda(), torch.from_numpy(rv).cuda(), d_dev)
    con.run(torch.from_numpy(lv).cuda(), torch.from_numpy(rv).cuda(), d_dev)      # accumulates twice
    torch.cuda.synchronize()
    l64, r64 = lv.astype(np.float64), rv.astype(np.float64)
    ref = _oracle_ref(lay, l64, r64, _oracle_ref(lay, l64, r64, dv.astype(np.float64)))
    bound = _oracle_ref(lay, np.abs(l64), np.abs(r64), np.zeros_like(ref))         # sum_k |l||r|
    eps = np.finfo(npdt).eps
    err = np.abs(d_dev.cpu().numpy().astype(np.float64) - ref)
    assert np.all(err <= 2 * 8 * lay.k * eps * bound + 8 * eps * np.abs(ref) + 1e-300), float(err.max())
