"""GPU parity for the diagonal property (the set {lowerTri, upperTri}; Sec. 2 "Matrix
Attribute"): scaling passes from either side, diagonal results, chains that mix diagonal
factors with every other property, transposed operands, the batched kernel."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import D, G, I, L, TOL, U, check_against_dense, eval_chain, rel_fro
from helpers import all_preorder_trees

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n", [1, 33, 130, 256, 300])
def test_diagonal_times_every_property_from_both_sides(n):
    for other in (G, L, U, D):
        for side in (0, 1):
            props = [D, other] if side == 0 else [other, D]
            if other == G:
                dims = [n, n, max(n - 5, 1)] if side == 0 else [n + 7, n, n]
            else:
                dims = [n, n, n]
            for flags in (0, mom.MOM_OUT_ZERO_FILL_TRIANGLE):
                plan, _ = check_against_dense(dims, props, sc.make_chain(dims, props, 2200 + n), flags=flags)
                assert plan.result[2] == other
                assert plan.cost_mults == oracle.tree_cost(dims, props, [0])[0]


def test_diagonal_with_transposed_and_strided_operands():
    n = 200
    for props, trans in (([D, L], [1, 1]), ([G, D], [1, 0]), ([D, G], [0, 1]), ([U, D], [1, 1])):
        dims = [n, n, n]
        f = sc.make_chain(dims, props, 2300, trans=trans)
        check_against_dense(dims, props, f, trans=trans, pad_cols=5, out_pad=3)
        check_against_dense(dims, props, f, trans=trans, pad_cols=4, out_pad=4)


def test_chains_with_diagonal_factors_every_tree():
    rng = np.random.default_rng(23)
    for trial in range(25):
        n = int(rng.integers(2, 6))
        props = [int(rng.choice([G, L, U, D, D, I])) for _ in range(n)]
        dims = [int(rng.choice([40, 70, 150]))]
        for p in props:
            dims.append(dims[-1] if p != G else int(rng.choice([40, 70, 150])))
        f = sc.make_chain(dims, props, 2400 + trial)
        plan, _ = check_against_dense(dims, props, f, flags=int(rng.integers(0, 2)))
        want = oracle.plan_bruteforce(dims, props)
        assert (plan.cost_mults, plan.splits) == (want["cost"], want["splits"])
        surv = oracle.survivors(props)
        if 3 <= len(surv) <= 4:
            for tree in all_preorder_trees(0, len(surv) - 1):
                check_against_dense(dims, props, f, splits=[surv[s] for s in tree])


def test_single_diagonal_factor_copies_only_the_diagonal():
    d = sc.make_factor(50, 50, D, 3)
    plan, got = eval_chain([50, 50, 50], [D, I], [d, None])
    assert plan.result == (50, 50, D)
    eye = np.eye(50, dtype=bool)
    assert np.array_equal(got[eye], d.numpy()[eye]) and np.all(np.isnan(got[~eye]))


def test_batched_chains_with_diagonal_factors():
    batch = 21
    for dims, props in (([32, 32, 32, 32], [D, G, U]), ([32, 32, 32, 32], [L, D, D]), ([32, 32, 17], [D, G])):
        host = sc.make_chain(dims, props, 2500, batch=batch)
        plan = mom.mom_chain_plan(dims, props)
        out = mom.mom_chain_eval_batched(plan, [f.cuda() for f in host])
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for b in range(batch):
            want = oracle.eval_dense(dims, props, [f[b].numpy() for f in host])
            assert rel_fro(got[b], want) <= TOL


def test_large_scaling_pass_whole_result():
    n = 4096
    dims, props = [n, n, n], [D, G]
    host = sc.make_chain(dims, props, 2600)
    plan, got = eval_chain(dims, props, host)
    dv = np.diag(host[0].numpy()).astype(np.float64)
    want = dv[:, None] * host[1].numpy().astype(np.float64)
    assert rel_fro(got, want) <= TOL
