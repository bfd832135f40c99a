"""GPU parity of the batched small-chain kernel (one launch for the whole batch)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, I, L, TOL, U, rel_fro

pytestmark = pytest.mark.gpu


def run_batched(dims, props, batch, family, splits=None):
    host = sc.make_chain(dims, props, family, batch=batch)
    plan = mom.mom_chain_plan(dims, props) if splits is None else mom.mom_plan_from_splits(dims, props, splits)
    dev = []
    for f, p in zip(host, props):
        if f is None:
            dev.append(None)
            continue
        d = f.cuda()
        if p in (L, U):          # the zero half must never be read
            keep = torch.tril(torch.ones_like(d[0], dtype=torch.bool)) if p == L else torch.triu(torch.ones_like(d[0], dtype=torch.bool))
            d = torch.where(keep, d, torch.full_like(d, float("nan")))
        dev.append(d.contiguous())
    rows, cols, prop = plan.result
    out = torch.full((batch, rows, cols), float("nan"), device="cuda", dtype=torch.float32)
    mom.mom_chain_eval_batched(plan, dev, out=out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not np.any(np.isnan(got))
    worst = 0.0
    for b in range(batch):
        want = oracle.eval_dense(dims, props, [None if f is None else f[b].numpy() for f in host])
        worst = max(worst, rel_fro(got[b], want))
    assert worst <= TOL, "worst chain: %.3e" % worst
    return plan, got


def test_workload_batched32_full_size():
    c = sc.CONFIGS["batched32"]
    plan, _ = run_batched(c.dims, c.props, c.batch, c.number)
    assert plan.string == "(0 (1 2))" and plan.cost_mults == 33792


def test_batched_other_tree_gives_the_same_values():
    c = sc.CONFIGS["batched32"]
    _, a = run_batched(c.dims, c.props, 257, c.number)
    plan, b = run_batched(c.dims, c.props, 257, c.number, splits=[1, 0])
    assert plan.string == "((0 1) 2)"
    assert rel_fro(a, b) <= 2 * TOL


@pytest.mark.parametrize("dims,props", [
    ([32, 32, 32], [L, L]), ([32, 32, 32], [U, U]), ([32, 32, 32], [G, G]),
    ([7, 19, 19, 3], [G, U, G]), ([31, 31, 31, 31, 5], [L, I, U, G]),
    ([5, 5, 5], [L, L]), ([1, 32, 1], [G, G]), ([30, 2, 17, 32, 32, 9], [G, G, G, L, G]),
    ([8] * 9, [G, L, U, G, L, U, G, L]), ([12, 12], [U]), ([20, 20, 20], [I, I]),
    ([6, 4], [G]),
])
def test_batched_shapes_and_properties(dims, props):
    run_batched(dims, props, 19, 7)


def test_batched_register_path_every_property_triple():
    # three full 32x32 factors multiplied as X0 (X1 X2) take the register-only kernel, which is
    # compiled once per property triple
    for p0 in (G, L, U):
        for p1 in (G, L, U):
            for p2 in (G, L, U):
                plan, _ = run_batched([32] * 4, [p0, p1, p2], 6, 40 + 9 * p0 + 3 * p1 + p2, splits=[0, 1])
                assert plan.string == "(0 (1 2))"


def test_batched_every_tree():
    from helpers import all_preorder_trees
    dims, props = [32, 32, 16, 32, 32], [U, G, G, L]
    for tree in all_preorder_trees(0, 3):
        plan, _ = run_batched(dims, props, 5, 3, splits=list(tree))
        assert plan.cost_mults == oracle.tree_cost(dims, props, list(tree))[0]


def test_batched_limits():
    p = mom.mom_chain_plan([33, 33, 33], [G, G])
    f = [torch.zeros(2, 33, 33, device="cuda") for _ in range(2)]
    with pytest.raises(mom.MomError):
        mom.mom_chain_eval_batched(p, f)
