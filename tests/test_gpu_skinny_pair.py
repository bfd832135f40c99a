"""GPU parity of the fused launch for (X * Y) * Z with a narrow intermediate: the plan keeps
both products (the multiplication count and the tree are untouched), the evaluation runs them
in one launch.  Whole results against the dense f64 oracle, aligned and ragged shapes."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, L, TOL, assert_close_by_tiles, check_against_dense, upload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("m,k1,w,n", [
    (8192, 512, 64, 2048),      # the shape inside the five-factor workload: no bounds checks at all
    (6144, 64, 64, 256),        # smallest that qualifies: one batch of k-groups, one pair per wavefront
    (6144, 2048, 64, 1024),     # many batches per wavefront
    (6200, 515, 50, 300),       # ragged everywhere: rows, k, width below 64, columns
    (7000, 40, 8, 257),         # narrowest intermediate, odd columns (unaligned result rows)
    (6144, 100, 33, 320),       # second 32-column block of the intermediate almost empty
])
def test_pair_launch_whole_result(m, k1, w, n):
    dims, props = [m, k1, w, n], [G, G, G]
    host = sc.make_chain(dims, props, 3300 + w)
    plan = mom.mom_plan_from_splits(dims, props, [1, 0])
    assert plan.string == "((0 1) 2)"
    assert mom.mom_plan_num_products(plan) == 2 and mom.mom_plan_num_launches(plan) == 1
    assert plan.cost_mults == oracle.tree_cost(dims, props, [1, 0])[0]
    dev = upload(host, props)
    out = torch.full((m, n), float("nan"), device="cuda")
    mom.mom_chain_eval(plan, dev, out=out)
    torch.cuda.synchronize()
    want = oracle.eval_dense(dims, props, [f.numpy() for f in host])
    assert_close_by_tiles(out.cpu().numpy(), want, G)


def test_pair_launch_with_strided_buffers_and_inside_a_longer_chain():
    # padded rows on every buffer; then the pair as the top of a five-factor tree
    dims, props = [6400, 96, 48, 512], [G, G, G]
    check_against_dense(dims, props, sc.make_chain(dims, props, 3400), splits=[1, 0], pad_cols=4, out_pad=4)
    check_against_dense(dims, props, sc.make_chain(dims, props, 3401), splits=[1, 0], pad_cols=3, out_pad=1)
    c = sc.CONFIGS["general5"]
    plan = mom.mom_chain_plan(c.dims, c.props)
    assert plan.string == "((0 (1 2)) (3 4))" and mom.mom_plan_num_launches(plan) == 3


def test_shapes_that_do_not_qualify_keep_their_two_launches():
    for dims, props in (([4096, 512, 64, 2048], [G, G, G]),        # too few row blocks
                        ([8192, 512, 65, 2048], [G, G, G]),        # intermediate too wide
                        ([8192, 512, 64, 128], [G, G, G]),         # second product too narrow
                        ([8192, 8192, 64, 2048], [L, G, G])):      # a triangular operand
        plan = mom.mom_plan_from_splits(dims, props, [1, 0])
        assert mom.mom_plan_num_launches(plan) >= 2
