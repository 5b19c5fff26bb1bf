"""The entry point that allocates nothing (tperm_execute_verified_static), called through the
C ABI and compared with the workspace form it is a variant of (tperm_execute_verified): same
transposed tensor bit for bit (and equal to the CPU oracle's), same verdict, on two calls in a
row of which the second has the smaller input; the device's free memory does not move across a
call; volumes beyond the stated maximum are refused before anything is launched."""
import ctypes

import numpy as np
import pytest

import oracle
from paper_1705_01598_amd import binding as B
from paper_1705_01598_amd import workloads as wl

pytestmark = pytest.mark.gpu
torch = pytest.importorskip("torch")
from gpu_util import GuardedOut, np_uint, to_device  # noqa: E402


def _both_forms(dims, perm, elem, seed):
    """Runs the workspace form and the static form on the same input; returns what they wrote."""
    L = B.lib()
    case = wl.make_case(0, seed, dims, perm, elem)
    a = wl.bitpattern_values(case)
    a_dev = to_device(a)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    plan = B.tperm_plan_create(dims, perm, elem)
    ref = oracle.transpose(a, dims, perm)
    # existing entry point: caller-owned workspace
    out_ws = GuardedOut(case.volume, elem)
    verdict_ws = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    nws = B.verify_workspace_bytes(case.volume)
    ws = torch.empty(nws // 8, dtype=torch.int64, device="cuda")
    st = L.tperm_execute_verified(plan.handle, ctypes.c_void_p(a_dev.data_ptr()), ctypes.c_void_p(out_ws.ptr), stream,
                                  ctypes.c_void_p(verdict_ws.data_ptr()), ctypes.c_void_p(ws.data_ptr()), nws)
    assert st == B.OK, B.status_string(st)
    # the variant that allocates nothing: no workspace argument
    out_st = GuardedOut(case.volume, elem)
    verdict_st = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    st = L.tperm_execute_verified_static(plan.handle, ctypes.c_void_p(a_dev.data_ptr()), ctypes.c_void_p(out_st.ptr),
                                         stream, ctypes.c_void_p(verdict_st.data_ptr()))
    assert st == B.OK, B.status_string(st)
    torch.cuda.synchronize()
    free_after = torch.cuda.mem_get_info()[0]
    got_ws, got_st = np_uint(out_ws.view().cpu().numpy()), np_uint(out_st.view().cpu().numpy())
    assert np.array_equal(got_st, got_ws), "the two forms wrote different tensors"
    assert np.array_equal(got_st, ref), "the static form differs from the oracle"
    assert out_ws.guards_intact() and out_st.guards_intact()
    assert int(verdict_ws.item()) == 0 and int(verdict_st.item()) == 0
    return free_before, free_after


def test_static_form_matches_workspace_form_twice_in_a_row_second_smaller():
    # first call: 1,386,000 elements of 8 bytes = 85 chunks of partial results per tensor
    _both_forms((70, 45, 33, 6, 2), (2, 0, 4, 3, 1), 8, 1)
    # second call, smaller (34,155 elements of 4 bytes = 3 chunks): the library's array still
    # holds the first call's partial results behind the three slots this call uses
    before, after = _both_forms((45, 33, 23), (2, 0, 1), 4, 2)
    assert before == after, "device memory in use changed across a call that must allocate nothing"
    # and once more with a larger one after the small one
    before, after = _both_forms((257, 129, 31), (1, 2, 0), 8, 3)
    assert before == after


def test_static_form_refuses_volumes_beyond_its_array():
    L = B.lib()
    dims, perm, elem = (16384, 8193), (1, 0), 4           # 2^27 + 16384 elements, 512 MiB + 64 KiB per tensor
    assert dims[0] * dims[1] > B.VERIFY_STATIC_MAX_ELEMS
    plan = B.tperm_plan_create(dims, perm, elem)
    a = torch.zeros(dims[0] * dims[1], dtype=torch.int32, device="cuda")
    out = torch.full((dims[0] * dims[1],), 7, dtype=torch.int32, device="cuda")
    verdict = torch.full((1,), 99, dtype=torch.int64, device="cuda")
    st = L.tperm_execute_verified_static(plan.handle, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream),
                                         ctypes.c_void_p(verdict.data_ptr()))
    torch.cuda.synchronize()
    assert st == B.ERR_TOO_LARGE
    assert int(verdict.item()) == 99 and bool((out == 7).all())          # nothing was launched
    # the largest volume it takes: exactly 2^27 elements
    dims = (16384, 8192)
    plan = B.tperm_plan_create(dims, perm, elem)
    a = torch.arange(dims[0] * dims[1], dtype=torch.int32, device="cuda")
    st = L.tperm_execute_verified_static(plan.handle, ctypes.c_void_p(a.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream),
                                         ctypes.c_void_p(verdict.data_ptr()))
    torch.cuda.synchronize()
    assert st == B.OK and int(verdict.item()) == 0
    assert torch.equal(out[:dims[0] * dims[1]].view(dims[0], dims[1]), a.view(dims[1], dims[0]).t())


def test_static_form_null_arguments():
    L = B.lib()
    plan = B.tperm_plan_create((4, 5), (1, 0), 8)
    x = ctypes.c_void_p(0x1000)
    assert L.tperm_execute_verified_static(None, x, x, None, x) == B.ERR_NULL
    assert L.tperm_execute_verified_static(plan.handle, x, ctypes.c_void_p(0x2000), None, None) == B.ERR_NULL
