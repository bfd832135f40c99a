"""GPU parity at the full workload sizes, in the launch configuration the benchmark times.
The dense oracle is out of reach here, so sampled rows are computed one by one by the oracle
(row r of the chain = row r of the first factor pushed through the others)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, I, L, TOL, U, rel_fro, structure_mask, upload

pytestmark = pytest.mark.gpu


def sample_rows(rows: int, seed: int, count: int = 12):
    rng = np.random.default_rng(seed)
    picks = {0, rows - 1, rows // 2, 127, 128} | {int(x) for x in rng.integers(0, rows, size=count)}
    return sorted(r for r in picks if 0 <= r < rows)


def run_and_check(name, splits=None, flags=0, expect_plan=None):
    c = sc.CONFIGS[name]
    host = sc.make_config(name)
    plan = mom.mom_chain_plan(c.dims, c.props) if splits is None else mom.mom_plan_from_splits(c.dims, c.props, splits)
    if expect_plan:
        assert plan.string == expect_plan
    want_plan = oracle.plan_bruteforce(c.dims, c.props)
    if splits is None:
        assert (plan.cost_mults, plan.splits) == (want_plan["cost"], want_plan["splits"])
    else:
        assert plan.cost_mults == oracle.tree_cost(c.dims, c.props, splits)[0]
    dev = upload(host, c.props, poison=True)
    rows, cols, prop = plan.result
    out = torch.full((rows, cols), float("nan"), device="cuda", dtype=torch.float32)
    ws = torch.full((max(plan.workspace_bytes, 4) // 4,), float("nan"), device="cuda", dtype=torch.float32)
    mom.mom_chain_eval(plan, dev, out=out, workspace=ws, flags=flags)
    torch.cuda.synchronize()
    picks = sample_rows(rows, c.number)
    got = out[picks].cpu().numpy()
    want = oracle.eval_rows(c.dims, c.props, [None if f is None else f.numpy() for f in host], picks)
    assert not np.any(np.isnan(got))
    for r, g, w in zip(picks, got, want):
        err = rel_fro(g, w)
        assert err <= TOL, "row %d: relative error %.3e" % (r, err)
    assert rel_fro(got, want) <= TOL
    # any size: nothing unwritten anywhere in a general result
    assert not bool(torch.isnan(out).any())
    return plan, out


def test_workload_trmm4096():
    run_and_check("trmm4096", expect_plan="(0 1)")


def test_workload_general5_planned_and_left_to_right():
    plan, a = run_and_check("general5", expect_plan="((0 (1 2)) (3 4))")
    c = sc.CONFIGS["general5"]
    plan2, b = run_and_check("general5", splits=oracle.left_to_right_splits(c.props),
                             expect_plan="((((0 1) 2) 3) 4)")
    assert plan2.cost_mults == 109521666048
    num = torch.linalg.norm((a - b).double()) / torch.linalg.norm(a.double())
    assert float(num) <= 2 * TOL


def test_workload_mixed5_planned():
    run_and_check("mixed5", expect_plan="(0 (2 (3 4)))")


def test_workload_mixed5_forced_triangular_intermediate():
    run_and_check("mixed5", splits=[2, 0, 3], expect_plan="((0 2) (3 4))")


def test_workload_mixed5_forced_left_to_right():
    run_and_check("mixed5", splits=[3, 2, 0], expect_plan="(((0 2) 3) 4)")


def test_lower_times_lower_8192_writes_only_the_triangle():
    n = 8192
    dims, props = [n, n, n], [L, L]
    host = sc.make_chain(dims, props, 40)
    plan = mom.mom_chain_plan(dims, props)
    assert plan.result == (n, n, L)
    dev = upload(host, props, poison=True)
    out = torch.full((n, n), float("nan"), device="cuda", dtype=torch.float32)
    mom.mom_chain_eval(plan, dev, out=out)
    torch.cuda.synchronize()
    nan = torch.isnan(out)
    upper = torch.triu(torch.ones(n, n, dtype=torch.bool, device="cuda"), 1)
    assert bool(torch.equal(nan, upper))                    # exactly the strict upper half untouched
    picks = sample_rows(n, 8)
    want = oracle.eval_rows(dims, props, [f.numpy() for f in host], picks)
    got = out[picks].cpu().numpy()
    for r, g, w in zip(picks, got, want):
        assert rel_fro(g[: r + 1], w[: r + 1]) <= TOL
