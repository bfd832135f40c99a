"""GPU side of the opt-in time objective (MOM_PLAN_MIN_TIME): the tree it picks evaluates to the
same values as the multiplication-optimal one and, on a chain where the two objectives part,
runs measurably faster."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, L, TOL, U, assert_close_by_tiles, upload

pytestmark = pytest.mark.gpu


def timed(call, reps=30):
    for _ in range(10):
        call()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    a.record()
    for _ in range(reps):
        call()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


def test_time_objective_tree_is_correct_and_faster_where_the_objectives_part():
    c = sc.CONFIGS["uug2048"]
    host = sc.make_config("uug2048")
    np_f = [f.numpy() for f in host]
    by_mults = mom.mom_chain_plan(c.dims, c.props)
    by_time = mom.mom_chain_plan_ex(c.dims, c.props, None, objective=mom.MOM_PLAN_MIN_TIME)
    want_t = oracle.plan_bruteforce_time(c.dims, c.props)
    assert (by_time.splits, by_time.cost_time_ps) == (want_t["splits"], want_t["time_ps"])
    assert by_mults.string == "((0 1) 2)" and by_time.string == "(0 (1 2))"
    assert by_time.cost_mults > by_mults.cost_mults and by_time.cost_time_ps < by_mults.cost_time_ps
    dev = upload(host, c.props, poison=True)
    want = oracle.eval_dense(c.dims, c.props, np_f)
    ms = {}
    for name, plan in (("mults", by_mults), ("time", by_time)):
        call = mom.bind_chain_eval(plan, dev)
        call.out.fill_(float("nan"))
        call()
        torch.cuda.synchronize()
        assert_close_by_tiles(call.out.cpu().numpy(), want, G)
        ms[name] = timed(call)
    assert ms["time"] < 0.9 * ms["mults"], ms


def test_time_objective_on_random_chains_matches_the_oracle_values():
    rng = np.random.default_rng(12)
    pool = [33, 64, 96, 130, 256, 300]
    for trial in range(12):
        n = int(rng.integers(2, 6))
        props = [int(rng.choice([G, G, L, U])) for _ in range(n)]
        dims = [int(rng.choice(pool))]
        for q in props:
            dims.append(dims[-1] if q != G else int(rng.choice(pool)))
        host = sc.make_chain(dims, props, 2100 + trial)
        plan = mom.mom_chain_plan_ex(dims, props, None, objective=mom.MOM_PLAN_MIN_TIME)
        out = mom.mom_chain_eval(plan, upload(host, props, poison=True), flags=mom.MOM_OUT_ZERO_FILL_TRIANGLE)
        torch.cuda.synchronize()
        want = oracle.eval_dense(dims, props, [f.numpy() for f in host])
        assert_close_by_tiles(out.cpu().numpy(), want, G)
