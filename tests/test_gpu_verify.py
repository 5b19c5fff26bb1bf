"""The self-checking execute (tperm_execute_verified) and its checking step on its own
(tperm_multiset_compare), through the C ABI.  The transposed tensor is compared with the CPU
oracle bit for bit as everywhere; the verdict word must be 0 for it.  The checking step is fed
buffers whose relation is known by construction: a permutation of the same words (equal), one
flipped bit, one word replaced by a copy of another, two words changed so that their plain sum
is unchanged."""
import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B
from paper_1705_01598_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
from gpu_util import GuardedOut, np_uint, to_device  # noqa: E402


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _compare(a_np, b_np, elem, offset_words=0):
    """verdict of tperm_multiset_compare on two host arrays of unsigned words."""
    n = a_np.size
    dt = torch.int64 if elem == 8 else torch.int32
    sign = np.int64 if elem == 8 else np.int32
    a = torch.zeros(n + offset_words, dtype=dt, device="cuda")
    b = torch.zeros(n + offset_words, dtype=dt, device="cuda")
    a[offset_words:] = torch.from_numpy(a_np.view(sign)).cuda()
    b[offset_words:] = torch.from_numpy(b_np.view(sign)).cuda()
    verdict = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.verify_workspace_bytes(n) // 8, dtype=torch.int64, device="cuda")
    B.tperm_multiset_compare(a.data_ptr() + offset_words * elem, b.data_ptr() + offset_words * elem, n, elem,
                             verdict.data_ptr(), ws.data_ptr(), ws.numel() * 8, _stream())
    torch.cuda.synchronize()
    return int(verdict.item())


@pytest.mark.parametrize("elem", [8, 4])
@pytest.mark.parametrize("n", [1, 2, 255, 16384, 16385, 50000, 1_000_003])
def test_multiset_compare_known_relations(n, elem):
    rng = np.random.default_rng(n * 10 + elem)
    dt = np.uint64 if elem == 8 else np.uint32
    a = rng.integers(0, np.iinfo(dt).max, size=n, dtype=dt, endpoint=True)
    assert _compare(a, a.copy(), elem) == 0
    assert _compare(a, rng.permutation(a), elem) == 0                       # same words, other places
    assert _compare(a, rng.permutation(a), elem, offset_words=1) == 0       # base pointers aligned to one word only
    flipped = a.copy()
    flipped[int(rng.integers(0, n))] ^= dt(1) << dt(int(rng.integers(0, 8 * elem)))
    assert _compare(a, flipped, elem) != 0                                  # one bit
    if n >= 2:
        i, j = (int(x) for x in rng.choice(n, size=2, replace=False))
        dup = a.copy()
        dup[i] = dup[j]
        if a[i] != a[j]:
            assert _compare(a, dup, elem) != 0                              # one word lost, another doubled
        bal = a.copy()                                                      # plain sum unchanged
        bal[i] = bal[i] + dt(12345)
        bal[j] = bal[j] - dt(12345)
        v = _compare(a, bal, elem)
        assert v != 0 and (v & 1) == 0 and (v & 4) != 0                     # the scrambled sum still sees it


CASES = [((70, 45, 33, 6), (2, 0, 3, 1), 8), ((8, 8, 8, 8, 8), (1, 3, 0, 2, 4), 4), ((5001, 477), (1, 0), 4),
         ((129, 1000), (0, 1), 8), ((33, 5, 7, 16, 3), (0, 3, 1, 4, 2), 4), ((1,), (0,), 8)]


@pytest.mark.parametrize("dims,perm,elem", CASES)
def test_execute_verified_matches_oracle_and_reports_equal(dims, perm, elem):
    case = wl.make_case(0, 77, dims, perm, elem)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    out = GuardedOut(case.volume, elem)
    verdict = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    nws = B.verify_workspace_bytes(case.volume)
    ws = torch.full((nws // 8 + 4,), -1, dtype=torch.int64, device="cuda")           # 4 words of guard behind it
    plan = B.tperm_plan_create(dims, perm, elem)
    B.tperm_execute_verified(plan, a_dev.data_ptr(), out.ptr, _stream(), verdict.data_ptr(), ws.data_ptr(), nws)
    torch.cuda.synchronize()
    assert np.array_equal(np_uint(out.view().cpu().numpy()), oracle.transpose(a, dims, perm))
    assert out.guards_intact() and int(verdict.item()) == 0
    assert bool((ws[nws // 8:] == -1).all())                                        # nothing written past the workspace


def test_execute_verified_argument_errors_launch_nothing():
    dims, perm, elem = (64, 50, 9), (2, 0, 1), 8
    case = wl.make_case(0, 78, dims, perm, elem)
    a_dev = to_device(wl.bitpattern_values(case))
    out = GuardedOut(case.volume, elem)
    verdict = torch.full((2,), 99, dtype=torch.int64, device="cuda")
    nws = B.verify_workspace_bytes(case.volume)
    ws = torch.empty(nws // 8 + 1, dtype=torch.int64, device="cuda")
    plan = B.tperm_plan_create(dims, perm, elem)
    s = _stream()
    call = lambda v, w, wb: B.tperm_execute_verified(plan, a_dev.data_ptr(), out.ptr, s, v, w, wb)
    for args, status in [((verdict.data_ptr(), ws.data_ptr(), nws - 64), B.ERR_TOO_LARGE),
                         ((verdict.data_ptr() + 4, ws.data_ptr(), nws), B.ERR_ALIGN),
                         ((verdict.data_ptr(), ws.data_ptr() + 4, nws), B.ERR_ALIGN),
                         ((0, ws.data_ptr(), nws), B.ERR_NULL),
                         ((verdict.data_ptr(), 0, nws), B.ERR_NULL),
                         ((ws.data_ptr() + 8, ws.data_ptr(), nws), B.ERR_ALIAS),
                         ((verdict.data_ptr(), a_dev.data_ptr(), nws), B.ERR_ALIAS)]:
        with pytest.raises(B.TpermError) as e:
            call(*args)
        assert e.value.status == status
    torch.cuda.synchronize()
    assert bool((out.view() == out.sent).all()) and int(verdict[0].item()) == 99     # untouched
