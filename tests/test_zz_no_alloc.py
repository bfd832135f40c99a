"""The entry point that allocates nothing (mom_chain_eval_static) against mom_chain_eval:
same kernels and same order of summation, so the results must be bit-identical; two calls in a
row share the library's per-GPU array, the second with a smaller chain."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, L, U, TOL, rel_fro, upload

pytestmark = pytest.mark.gpu


def raw_static_call(plan, dev, out, flags=0):
    """Straight through the C ABI: pointers and sizes only."""
    lib = mom.library()
    n = plan.n
    ptrs = (ctypes.c_void_p * n)(*[None if f is None else f.data_ptr() for f in dev])
    st = lib.mom_chain_eval_static(plan.handle, ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p)), None,
                                   ctypes.c_void_p(out.data_ptr()), 0, flags,
                                   ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return st


def both_ways(dims, props, family, splits=None):
    host = sc.make_chain(dims, props, family)
    plan = mom.mom_chain_plan(dims, props) if splits is None else mom.mom_plan_from_splits(dims, props, splits)
    dev = upload(host, props, poison=True)
    rows, cols, prop = plan.result
    want = torch.full((rows, cols), float("nan"), device="cuda")
    mom.mom_chain_eval(plan, dev, out=want)
    got = torch.full((rows, cols), float("nan"), device="cuda")
    assert raw_static_call(plan, dev, got) == 0
    torch.cuda.synchronize()
    g, w = got.cpu().numpy(), want.cpu().numpy()
    assert np.array_equal(g, w, equal_nan=True), "static-workspace result differs from mom_chain_eval's"
    ref = oracle.eval_dense(dims, props, [None if f is None else f.numpy() for f in host])
    keep = ~np.isnan(w)
    assert rel_fro(np.where(keep, g, 0.0), np.where(keep, ref, 0.0)) <= TOL
    return plan


def test_static_workspace_two_calls_in_a_row_second_smaller():
    # temporaries of two levels plus split-K slices of two fused products, then a smaller chain
    # (other offsets, other slice counts) over the same array with the first call's leftovers in it
    p1 = both_ways([96, 1500, 80, 1200, 72], [G, G, G, G], 830, splits=[1, 0, 2])
    assert p1.workspace_bytes > 0
    p2 = both_ways([70, 70, 70, 40], [L, U, G], 831, splits=[1, 0])
    assert 0 < p2.workspace_bytes < p1.workspace_bytes
    p3 = both_ways([64, 5000, 64], [G, G], 832)                   # split-K only
    assert p3.workspace_bytes > 0


def test_static_workspace_limit_and_errors():
    n = 8192
    big = mom.mom_plan_from_splits([n] * 4, [G, G, G], [1, 0])       # one 256 MB temporary
    assert big.workspace_bytes > mom.MOM_STATIC_WORKSPACE_BYTES
    x = torch.zeros(8, device="cuda")
    lib = mom.library()
    fake = (ctypes.c_void_p * 3)(x.data_ptr(), x.data_ptr(), x.data_ptr())
    st = lib.mom_chain_eval_static(big.handle, ctypes.cast(fake, ctypes.POINTER(ctypes.c_void_p)), None,
                                   ctypes.c_void_p(x.data_ptr()), 0, 0, None)
    assert mom.binding.STATUS_NAMES[st] == "MOM_ERR_WORKSPACE"
    small = mom.mom_chain_plan([4, 4, 4], [G, G])
    fake2 = (ctypes.c_void_p * 2)(x.data_ptr(), x.data_ptr())
    st = lib.mom_chain_eval_static(small.handle, ctypes.cast(fake2, ctypes.POINTER(ctypes.c_void_p)), None,
                                   ctypes.c_void_p(x.data_ptr()), 0, 4, None)
    assert mom.binding.STATUS_NAMES[st] == "MOM_ERR_BAD_FLAGS"


def test_static_workspace_fits_the_mixed_property_workload():
    c = sc.CONFIGS["mixed5"]
    plan = mom.mom_chain_plan(c.dims, c.props)
    assert plan.workspace_bytes <= mom.MOM_STATIC_WORKSPACE_BYTES
