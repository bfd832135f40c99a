"""Host logic of the library (no GPU): planner against the oracle's brute force, error paths,
exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from helpers import golden_lines, random_chain

G, L, U, I = 0, 1, 2, 3
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mom.h")).read()
    declared = set(re.findall(r"\b(mom_[a-z_]+)\s*\(", header))
    declared -= {"mom_plan_t"}
    assert {"mom_chain_plan", "mom_chain_eval", "mom_chain_eval_batched", "mom_plan_from_splits"} <= declared
    lib = mom.library()
    for name in sorted(declared):
        assert hasattr(lib, name), name
    from paper_2208_10391_amd import binding
    assert set(binding.EXPORTS) == declared


def test_plans_equal_bruteforce_on_random_chains():
    rng = np.random.default_rng(2024)
    checked = 0
    for trial in range(6000):
        n = int(rng.integers(1, 10)) if trial % 10 else int(rng.integers(9, 11))
        if trial >= 3000:
            n = min(n, 7)
        dims, props = random_chain(rng, n, 40)
        want = oracle.plan_bruteforce(dims, props)
        plan = mom.mom_chain_plan(dims, props)
        assert plan.cost_mults == want["cost"], (dims, props)
        assert plan.splits == want["splits"], (dims, props)
        assert plan.string == oracle.plan_string(props, want["splits"])
        rows, cols, prop = plan.result
        assert (rows, cols, prop) == (dims[0], dims[-1], want["result_prop"])
        assert mom.mom_plan_num_products(plan) == max(want["n_eff"] - 1, 0)
        checked += 1
    assert checked == 6000


def test_plans_equal_bruteforce_with_few_distinct_dims():
    # few distinct sizes produce many exact ties: the tie-break must agree as well
    rng = np.random.default_rng(5)
    for _ in range(3000):
        n = int(rng.integers(2, 9))
        props = [int(rng.choice([G, G, L, U, I])) for _ in range(n)]
        sizes = [int(rng.choice([2, 4, 8]))]
        for p in props:
            sizes.append(sizes[-1] if p != G else int(rng.choice([2, 4, 8])))
        want = oracle.plan_bruteforce(sizes, props)
        plan = mom.mom_chain_plan(sizes, props)
        assert (plan.cost_mults, plan.splits) == (want["cost"], want["splits"]), (sizes, props)


def test_workload_plans():
    for ln in golden_lines("workload_plans.txt"):
        w = ln.split(" ", 5)
        c = sc.CONFIGS[w[1]]
        plan = mom.mom_chain_plan(c.dims, c.props)
        assert plan.cost_mults == int(w[3]) and plan.string == w[5]


def test_paper_sec4_chain_and_forced_initial_tree():
    kv = dict(ln.split(" ", 1) for ln in golden_lines("sec4_chain.txt"))
    dims = [int(x) for x in kv["dims"].split()]
    plan = mom.mom_chain_plan(dims, [G] * 4)
    assert plan.string == kv["chosen"] and plan.cost_mults == int(kv["chosen_mults"])
    forced = mom.mom_plan_from_splits(dims, [G] * 4, oracle.left_to_right_splits([G] * 4))
    assert forced.string == kv["initial"] and forced.cost_mults == int(kv["initial_mults"])


def test_forced_trees_cost_like_the_oracle():
    c = sc.CONFIGS["mixed5"]
    for splits, text in (([2, 0, 3], "((0 2) (3 4))"), ([3, 2, 0], "(((0 2) 3) 4)"), ([0, 2, 3], "(0 (2 (3 4)))")):
        plan = mom.mom_plan_from_splits(c.dims, c.props, splits)
        assert plan.string == text
        assert plan.cost_mults == oracle.tree_cost(c.dims, c.props, splits)[0]
        assert plan.splits == splits


def test_listing_5x5_plan():
    plan = mom.mom_chain_plan([5, 5, 5], [L, L])
    assert plan.cost_mults == 35 and plan.result == (5, 5, L) and plan.string == "(0 1)"
    assert plan.workspace_bytes == 0


def test_degenerate_chains():
    p = mom.mom_chain_plan([7, 7, 7], [I, I])
    assert (p.string, p.cost_mults, p.result, mom.mom_plan_num_products(p)) == ("I", 0, (7, 7, I), 0)
    p = mom.mom_chain_plan([7, 7, 7, 7], [I, U, I])
    assert (p.string, p.cost_mults, p.result, p.splits) == ("1", 0, (7, 7, U), [])
    p = mom.mom_chain_plan([3, 9], [G])
    assert (p.string, p.result) == ("0", (3, 9, G))


def test_workspace_reuses_released_temporaries():
    # right-nested chain of equal squares: two temporaries alternate, never more
    n, k = 64, 6
    plan = mom.mom_plan_from_splits([n] * (k + 1), [G] * k, list(range(k - 1)))
    assert plan.string == "(0 (1 (2 (3 (4 5)))))"
    assert plan.workspace_bytes == 2 * n * n * 4


def status_of(fn, *args):
    with pytest.raises(mom.MomError) as e:
        fn(*args)
    return e.value.status


def test_error_paths():
    names = __import__("paper_2208_10391_amd.binding", fromlist=["x"]).STATUS_NAMES
    code = {n: i for i, n in enumerate(names)}
    assert status_of(mom.mom_chain_plan, [4], []) == code["MOM_ERR_BAD_N"]
    assert status_of(mom.mom_chain_plan, [4, 0], [G]) == code["MOM_ERR_BAD_DIM"]
    assert status_of(mom.mom_chain_plan, [4, -3], [G]) == code["MOM_ERR_BAD_DIM"]
    assert status_of(mom.mom_chain_plan, [4, 2 ** 31], [G]) == code["MOM_ERR_BAD_DIM"]
    assert status_of(mom.mom_chain_plan, [4, 2 ** 31 - 255], [G]) == code["MOM_ERR_BAD_DIM"]
    assert mom.mom_chain_plan([4, 2 ** 31 - 256], [G]).cost_mults == 0       # the largest dimension allowed
    assert status_of(mom.mom_chain_plan, [4, 4], [7]) == code["MOM_ERR_BAD_PROP"]
    for p in (L, U, I):
        assert status_of(mom.mom_chain_plan, [4, 5], [p]) == code["MOM_ERR_NOT_SQUARE"]
    assert status_of(mom.mom_plan_from_splits, [4, 4, 4, 4], [G, G, G], [2, 0]) == code["MOM_ERR_BAD_SPLITS"]
    assert status_of(mom.mom_plan_from_splits, [4, 4, 4, 4], [G, G, G], [0, 0]) == code["MOM_ERR_BAD_SPLITS"]
    assert status_of(mom.mom_plan_from_splits, [4, 4, 4, 4], [G, I, G], [1]) == code["MOM_ERR_BAD_SPLITS"]
    assert status_of(mom.mom_plan_from_splits, [4, 4, 4, 4], [G, G, G], [0]) == code["MOM_ERR_BAD_SPLITS"]
    # the largest dimension cubed, three times over, does not fit in 64 bits
    big = 2 ** 31 - 256
    assert status_of(mom.mom_chain_plan, [big] * 5, [G] * 4) == code["MOM_ERR_OVERFLOW"]
    lib = mom.library()
    assert lib.mom_chain_plan(None, None, 1, None) == code["MOM_ERR_NULL"]
    out = ctypes.c_void_p(123)
    assert lib.mom_chain_plan(None, None, 1, ctypes.byref(out)) == code["MOM_ERR_NULL"] and not out.value
    p = mom.mom_chain_plan([4, 4, 4], [G, G])
    small = ctypes.create_string_buffer(3)
    assert lib.mom_plan_string(p.handle, small, 3) == code["MOM_ERR_BUFFER_TOO_SMALL"]
    assert lib.mom_plan_splits(p.handle, (ctypes.c_int32 * 1)(), 0) == code["MOM_ERR_BUFFER_TOO_SMALL"]
    # evaluation argument checks that need no GPU: nothing is launched on these paths
    assert lib.mom_chain_eval(p.handle, None, None, None, 0, None, 0, 0, None) == code["MOM_ERR_NULL"]
    assert lib.mom_chain_eval(None, None, None, None, 0, None, 0, 0, None) == code["MOM_ERR_NULL"]
    fake = (ctypes.c_void_p * 2)(256, 512)
    fptr = ctypes.cast(fake, ctypes.POINTER(ctypes.c_void_p))
    lds = (ctypes.c_int64 * 2)(3, 4)
    assert lib.mom_chain_eval(p.handle, fptr, lds, ctypes.c_void_p(1024), 0, None, 0, 0, None) == code["MOM_ERR_BAD_STRIDE"]
    assert lib.mom_chain_eval(p.handle, fptr, None, ctypes.c_void_p(1024), 2, None, 0, 0, None) == code["MOM_ERR_BAD_STRIDE"]
    p3 = mom.mom_chain_plan([4, 4, 4, 4], [G, G, G])
    fake3 = (ctypes.c_void_p * 3)(256, 512, 768)
    fptr3 = ctypes.cast(fake3, ctypes.POINTER(ctypes.c_void_p))
    assert p3.workspace_bytes > 0
    assert lib.mom_chain_eval(p3.handle, fptr3, None, ctypes.c_void_p(1024), 0, None, 0, 0, None) == code["MOM_ERR_WORKSPACE"]
    assert lib.mom_chain_eval(p3.handle, fptr3, None, ctypes.c_void_p(1024), 0, ctypes.c_void_p(4096), 8, 0, None) == code["MOM_ERR_WORKSPACE"]
    assert lib.mom_chain_eval(p3.handle, fptr3, None, ctypes.c_void_p(1024), 0, ctypes.c_void_p(4100), 1 << 20, 0, None) == code["MOM_ERR_WORKSPACE"]
    # unknown flag bits are refused, not ignored
    assert lib.mom_chain_eval(p.handle, fptr, None, ctypes.c_void_p(1024), 0, None, 0, 2, None) == code["MOM_ERR_BAD_FLAGS"]
    assert lib.mom_chain_eval(p.handle, fptr, None, ctypes.c_void_p(1024), 0, None, 0, 0x80000001, None) == code["MOM_ERR_BAD_FLAGS"]
    for name in ("MOM_ERR_NOMEM", "MOM_ERR_BAD_FLAGS", "MOM_ERR_NOT_READY"):
        assert mom.mom_status_string(code[name]) not in ("ok", "unknown status")
    pbig = mom.mom_chain_plan([33, 33, 33], [G, G])
    assert lib.mom_chain_eval_batched(pbig.handle, fptr, None, ctypes.c_void_p(1024), 0, 4, None) == code["MOM_ERR_UNSUPPORTED"]
    assert lib.mom_chain_eval_batched(p.handle, fptr, None, ctypes.c_void_p(1024), 0, -1, None) == code["MOM_ERR_BAD_N"]
    assert lib.mom_chain_eval_batched(p.handle, fptr, (ctypes.c_int64 * 2)(15, 16), ctypes.c_void_p(1024), 0, 4, None) == code["MOM_ERR_BAD_STRIDE"]
    assert mom.mom_status_string(0) == "ok" and "square" in mom.mom_status_string(code["MOM_ERR_NOT_SQUARE"])


def test_plans_with_transposed_factors_equal_bruteforce():
    # Table 1 Transpose; Sec. 2 Transformations: a transposed lowerTri factor plans as upperTri
    rng = np.random.default_rng(77)
    for trial in range(3000):
        n = int(rng.integers(1, 9))
        dims, props = random_chain(rng, n, 40)
        trans = [int(x) for x in rng.integers(0, 2, size=n)]
        want = oracle.plan_bruteforce(dims, props, trans=trans)
        plan = mom.mom_chain_plan(dims, props, trans=trans)
        assert (plan.cost_mults, plan.splits, plan.result[2]) == (want["cost"], want["splits"], want["result_prop"])
        assert plan.string == oracle.plan_string(props, want["splits"])
    p = mom.mom_chain_plan([5, 5, 5], [L, U], trans=[1, 0])
    assert p.result == (5, 5, U) and p.cost_mults == 35          # upper * upper
    p = mom.mom_chain_plan([5, 5, 5], [L, L], trans=[1, 0])
    assert p.result == (5, 5, G) and p.cost_mults == 55          # upper * lower: sum of squares
    p = mom.mom_chain_plan([4, 4, 4], [I, G], trans=[1, 1])
    assert p.result == (4, 4, G) and p.cost_mults == 0
    # forced tree through the general call
    p = mom.mom_chain_plan_ex([3, 4, 5, 6], [G, G, G], [1, 0, 1], preorder_splits=[0, 1])
    assert p.string == "(0 (1 2))"
    assert status_of(mom.mom_chain_plan, [4, 4, 4], [G, G], [0, 2]) == mom.binding.STATUS_NAMES.index("MOM_ERR_BAD_TRANS")
    assert status_of(mom.mom_chain_plan_ex, [4, 4, 4], [G, G], None, 9) == mom.binding.STATUS_NAMES.index("MOM_ERR_BAD_FLAGS")
    # strides are those of the STORED matrix: a transposed 3x7 factor is a 7x3 buffer
    lib = mom.library()
    p = mom.mom_chain_plan([3, 7, 2], [G, G], trans=[1, 0])
    fake = (ctypes.c_void_p * 2)(256, 512)
    fptr = ctypes.cast(fake, ctypes.POINTER(ctypes.c_void_p))
    bad = mom.binding.STATUS_NAMES.index("MOM_ERR_BAD_STRIDE")
    assert lib.mom_chain_eval(p.handle, fptr, (ctypes.c_int64 * 2)(2, 2), ctypes.c_void_p(1024), 0, None, 0, 0, None) == bad


def test_time_objective_equals_the_oracle_enumeration():
    """MOM_PLAN_MIN_TIME: the library's DP (closed-form chunk sums) against the oracle's exhaustive
    search over the same stated model (tile by tile): tree and picoseconds bit-exact."""
    rng = np.random.default_rng(55)
    pool = [1, 5, 31, 32, 33, 64, 65, 96, 127, 128, 129, 130, 200, 256, 300, 512, 1000, 2050, 4096]
    checked = 0
    for trial in range(2500):
        n = int(rng.integers(1, 8))
        props = [int(rng.choice([G, G, L, U, I])) for _ in range(n)]
        dims = [int(rng.choice(pool))]
        for q in props:
            dims.append(dims[-1] if q != G else int(rng.choice(pool)))
        trans = [int(x) for x in rng.integers(0, 2, size=n)] if trial % 3 == 0 else None
        want = oracle.plan_bruteforce_time(dims, props, trans=trans)
        plan = mom.mom_chain_plan_ex(dims, props, trans, objective=mom.MOM_PLAN_MIN_TIME)
        assert (plan.cost_time_ps, plan.splits, plan.cost_mults) == (want["time_ps"], want["splits"], want["mults"]), (dims, props)
        # the default objective is untouched, and any plan reports its modelled time
        base = mom.mom_chain_plan(dims, props, trans=trans)
        ref = oracle.plan_bruteforce(dims, props, trans=trans)
        assert (base.cost_mults, base.splits) == (ref["cost"], ref["splits"])
        assert base.cost_time_ps == oracle.tree_time_ps(dims, props, base.splits, trans=trans)
        assert base.cost_time_ps >= plan.cost_time_ps and base.cost_mults <= plan.cost_mults
        checked += 1
    assert checked == 2500
    # single products against the hand-worked values
    for m, k, n, px, py, want in ([int(x) for x in ln.split()] for ln in golden_lines("time_model.txt")):
        assert mom.mom_chain_plan([m, k, n], [px, py]).cost_time_ps == want
    # the workloads keep their trees under the time model
    for name in ("trmm4096", "general5", "mixed5"):
        c = sc.CONFIGS[name]
        a = mom.mom_chain_plan(c.dims, c.props)
        b = mom.mom_chain_plan_ex(c.dims, c.props, None, objective=mom.MOM_PLAN_MIN_TIME)
        assert a.splits == b.splits
    # and one chain where the objectives part (see tests/test_oracle_time_model.py)
    a = mom.mom_chain_plan([256, 1024, 4096, 256, 256], [G, G, G, L])
    b = mom.mom_chain_plan_ex([256, 1024, 4096, 256, 256], [G, G, G, L], None, objective=mom.MOM_PLAN_MIN_TIME)
    assert (a.string, b.string) == ("((0 (1 2)) 3)", "((0 1) (2 3))")


def test_plans_with_diagonal_factors_equal_bruteforce_under_both_objectives():
    D = 4
    rng = np.random.default_rng(91)
    pool = [1, 5, 32, 64, 65, 130, 256, 1000]
    for trial in range(2000):
        n = int(rng.integers(1, 8))
        props = [int(rng.choice([G, L, U, I, D, D])) for _ in range(n)]
        dims = [int(rng.choice(pool))]
        for q in props:
            dims.append(dims[-1] if q != G else int(rng.choice(pool)))
        want = oracle.plan_bruteforce(dims, props)
        plan = mom.mom_chain_plan(dims, props)
        assert (plan.cost_mults, plan.splits, plan.result[2]) == (want["cost"], want["splits"], want["result_prop"])
        wt = oracle.plan_bruteforce_time(dims, props)
        pt = mom.mom_chain_plan_ex(dims, props, None, objective=mom.MOM_PLAN_MIN_TIME)
        assert (pt.cost_time_ps, pt.splits, pt.cost_mults) == (wt["time_ps"], wt["splits"], wt["mults"])
    assert mom.mom_chain_plan([6, 6, 6], [D, D]).result == (6, 6, D)
    assert mom.mom_chain_plan([6, 6, 6], [D, I]).result == (6, 6, D)
    assert status_of(mom.mom_chain_plan, [6, 7], [D]) == mom.binding.STATUS_NAMES.index("MOM_ERR_NOT_SQUARE")
    assert status_of(mom.mom_chain_plan, [6, 6], [5]) == mom.binding.STATUS_NAMES.index("MOM_ERR_BAD_PROP")


def test_equation_plans_sum_property_cost_and_errors():
    # Table 1 Add / Equation: a sum of chains; every addend planned like a chain of its own
    D = 4
    rng = np.random.default_rng(101)
    for trial in range(300):
        n = int(rng.choice([1, 3, 8, 20]))
        k = int(rng.integers(1, 5))
        chains = []
        for c in range(k):
            length = int(rng.integers(1, 4))
            props = [int(rng.choice([G, L, U, I, D])) for _ in range(length)]
            trans = [int(x) for x in rng.integers(0, 2, size=length)]
            chains.append(([n] * (length + 1), props, trans))
        eq = mom.mom_equation_plan(chains)
        want_prop = oracle.equation_property([(d, p, None, t) for d, p, t in chains])
        assert eq.result == (n, n, want_prop)
        assert eq.cost_mults == sum(oracle.plan_bruteforce(d, p, trans=t)["cost"] for d, p, t in chains)
        for c, (d, p, t) in enumerate(chains):
            assert eq.chain_string(c) == oracle.plan_string(p, oracle.plan_bruteforce(d, p, trans=t)["splits"])
    # a pure variadic Add needs no workspace; a single product-bearing addend goes straight to the output
    assert mom.mom_equation_plan([([5, 5], [G], None)] * 4).workspace_bytes == 0
    assert mom.mom_equation_plan([([5, 5, 5], [G, G], None), ([5, 5], [G], None)]).workspace_bytes == 0
    two = mom.mom_equation_plan([([64, 64, 64], [G, G], None), ([64, 64, 64], [L, G], None)])
    assert two.workspace_bytes == 64 * 64 * 4
    code = {n: i for i, n in enumerate(mom.binding.STATUS_NAMES)}
    assert status_of(mom.mom_equation_plan, [([5, 5], [G], None), ([5, 6], [G], None)]) == code["MOM_ERR_BAD_DIM"]
    assert status_of(mom.mom_equation_plan, []) == code["MOM_ERR_BAD_N"]
    assert status_of(mom.mom_equation_plan, [([5, 6], [L], None)]) == code["MOM_ERR_NOT_SQUARE"]
    lib = mom.library()
    assert lib.mom_equation_eval(None, None, None, None, 0, None, 0, 0, None) == code["MOM_ERR_NULL"]
    assert lib.mom_equation_eval(two.handle, None, None, ctypes.c_void_p(1024), 0, None, 0, 0, None) == code["MOM_ERR_NULL"]
    fake = (ctypes.c_void_p * 4)(256, 512, 768, 1024)
    fptr = ctypes.cast(fake, ctypes.POINTER(ctypes.c_void_p))
    assert lib.mom_equation_eval(two.handle, fptr, None, ctypes.c_void_p(1024), 0, None, 0, 0, None) == code["MOM_ERR_WORKSPACE"]
    assert lib.mom_equation_eval(two.handle, fptr, None, ctypes.c_void_p(1024), 0, None, 0, 8, None) == code["MOM_ERR_BAD_FLAGS"]
    assert lib.mom_equation_eval(two.handle, fptr, None, ctypes.c_void_p(1024), 3, None, 0, 0, None) == code["MOM_ERR_BAD_STRIDE"]


def test_operands_of_a_shared_launch_stay_alive_until_it_runs():
    # ((((0 1) 2) 3) 4) of the five-factor workload: (T * A2) * A3 with T = A0 * A1 runs as one launch
    # that reads T while it writes its result, so T (256 MiB), the never-written 8192 x 64
    # intermediate (2 MiB) and the result (128 MiB) must not share workspace
    c = sc.CONFIGS["general5"]
    plan = mom.mom_plan_from_splits(c.dims, c.props, [3, 2, 1, 0])
    assert mom.mom_plan_num_launches(plan) == 3
    mib = 1 << 20
    assert plan.workspace_bytes >= (256 + 2 + 128) * mib
    levels = [mom.mom_plan_product(plan, i)["level"] for i in range(4)]
    assert levels == [1, 3, 3, 4]                 # the absorbed product stands at its consumer's level (3)


def test_launch_layout_of_the_chooser():
    """How many launches the planner lays out (host logic only): one per product or fused level,
    plus one slice-sum launch wherever tiles are cut along k."""
    cases = [
        ([4096, 4096, 4096], [L, G], 1),           # 1024 tiles in 512 pairs
        ([3072, 288, 3072], [G, G], 1),            # 576 equal tiles, k too short to cut the last round
        ([3072, 1024, 3072], [G, G], 2),           # 576 = 2.25 tiles per compute unit: last three tile rows cut along k
        ([6144, 1024, 6144], [G, G], 1),           # 2304 = 9 per compute unit: nothing to gain
        ([3328, 3328, 3328], [G, G], 1),           # a tail of 182 tiles is too large to be worth cutting
        ([64, 4096, 64], [G, G], 2),               # one small tile, long k: k-slices
        ([1024, 1024, 1024], [G, G], 1),           # 256 tiles of 64 x 64
        ([2048, 2048, 256], [L, G], 2),            # 128 small tiles, 64 chunks: k-slices
        ([2048, 2048, 2048], [L, L], 1),           # 528 small tiles
        ([8192, 512, 8192, 64, 4096, 2048], [G] * 5, 3),      # two products and their slice sum, then (X Y) Z in one
        ([256, 1024, 4096, 256, 256], [G, G, G, L], 4),
    ]
    for dims, props, want in cases:
        plan = mom.mom_chain_plan(dims, props)
        assert mom.mom_plan_num_launches(plan) == want, (dims, props, mom.mom_plan_num_launches(plan))
        # the workspace covers the slices: never smaller than the temporaries alone
        assert plan.workspace_bytes >= 0
