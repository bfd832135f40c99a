"""GPU side of the opt-in time objective (MOM_PLAN_MIN_TIME): the tree it picks evaluates to the
same values as the multiplication-optimal one and, on a chain where the two objectives part,
runs measurably faster."""
import itertools

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
    c = sc.CONFIGS["gggl256"]
    host = sc.make_config("gggl256")
    np_f = [f.numpy() for f in host]
    by_mults = mom.mom_chain_plan(c.dims, c.props)
    by_time = mom.mom_chain_plan_ex(c.dims, c.props, None, objective=mom.MOM_PLAN_MIN_TIME)
    want_t = oracle.plan_bruteforce_time(c.dims, c.props)
    assert (by_time.splits, by_time.cost_time_ps) == (want_t["splits"], want_t["time_ps"])
    assert by_mults.string == "((0 (1 2)) 3)" and by_time.string == "((0 1) (2 3))"
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
        ms[name] = min(timed(call) for _ in range(3))
    assert ms["time"] < 0.9 * ms["mults"], ms


def test_wherever_the_objectives_part_the_time_tree_is_the_faster_one():
    """Every chain of three or four factors with dimensions from a pool of powers of two and
    properties general / lowerTri / upperTri on which the two objectives choose different trees
    with a modelled gain of at least 8 % (and at least 40 us, so that the difference is not
    launch noise): both trees are timed.  The model is an estimate: the bar is that its tree
    wins on nine chains out of ten and never loses by more than 8 % (the worst seen: 5.6 % on
    G.G.U.G 256 x 4096 x 2048 x 2048 x 256, where the model prefers three dependent products to two
    independent ones and a root)."""
    pool = [64, 128, 256, 512, 1024, 2048, 4096]
    parted = []
    for n in (3, 4):
        for props in itertools.product([G, L, U], repeat=n):
            if n == 4 and all(q == G for q in props):
                continue
            for dims in itertools.product(pool, repeat=n + 1):
                if max(dims) < 1024 or any(q != G and dims[t] != dims[t + 1] for t, q in enumerate(props)):
                    continue
                if sum(dims[t] * dims[t + 1] for t in range(n)) * 4 > 600e6:
                    continue
                a = mom.mom_chain_plan(dims, props)
                b = mom.mom_chain_plan_ex(dims, props, None, objective=mom.MOM_PLAN_MIN_TIME)
                if a.splits != b.splits and a.cost_time_ps >= 40e6 and a.cost_time_ps >= 1.08 * b.cost_time_ps:
                    parted.append((list(dims), list(props), a, b))
    assert len(parted) >= 10, "the family should contain chains on which the objectives part"
    faster, worst = 0, (0.0, None)
    for dims, props, a, b in parted:
        dev = [f.cuda() for f in sc.make_chain(dims, props, 2300)]
        call_a, call_b = mom.bind_chain_eval(a, dev), mom.bind_chain_eval(b, dev)
        ta = tb = float("inf")
        for _ in range(3):                       # in turn, best of three: clock ramps and stray stalls cancel
            ta, tb = min(ta, timed(call_a)), min(tb, timed(call_b))
        faster += tb < ta
        if tb / ta > worst[0]:
            worst = (tb / ta, (dims, props, a.string, b.string, ta, tb))
        del dev
        torch.cuda.empty_cache()
    assert faster >= 0.9 * len(parted), (faster, len(parted), worst)
    assert worst[0] <= 1.08, worst


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
