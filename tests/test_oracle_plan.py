"""Pins for the oracle's planner side: cost unit, closed forms, brute-force optimum."""
import numpy as np
import pytest

import oracle
from helpers import all_preorder_trees, golden_lines, random_chain

G, L, U, I = 0, 1, 2, 3


def pattern(prop, r, c):
    ones = np.ones((r, c), dtype=np.int64)
    return {G: ones, L: np.tril(ones), U: np.triu(ones), I: np.eye(r, c, dtype=np.int64)}[prop]


def shape_for(pX, pY, m, k, n):
    if pX != G:
        m = k
    if pY != G:
        n = k
    return m, k, n


@pytest.mark.parametrize("pX", [G, L, U, I])
@pytest.mark.parametrize("pY", [G, L, U, I])
def test_count_mults_equals_pattern_product(pX, pY):
    # number of (i,t,j) with both operands structurally non-zero = sum of the 0/1 pattern product
    for k in range(1, 13):
        m, k, n = shape_for(pX, pY, k + 2, k, k + 3)
        want = int((pattern(pX, m, k) @ pattern(pY, k, n)).sum())
        assert oracle.count_mults(m, k, n, pX, pY) == want


def closed_form(pX, pY, m, k, n):
    tri = (L, U)
    if pX == G and pY == G:
        return m * k * n
    if pX in tri and pY == G:
        return n * m * (m + 1) // 2
    if pX == G and pY in tri:
        return m * n * (n + 1) // 2
    if pX == pY:
        return n * (n + 1) * (n + 2) // 6
    return n * (n + 1) * (2 * n + 1) // 6


@pytest.mark.parametrize("pX", [G, L, U])
@pytest.mark.parametrize("pY", [G, L, U])
def test_closed_form_costs_match_counted_mults(pX, pY):
    # the oracle's own cost of a two-factor chain must be the counted number of products
    for k in range(1, 13):
        m, k, n = shape_for(pX, pY, k + 1, k, k + 4)
        counted = oracle.count_mults(m, k, n, pX, pY)
        assert counted == closed_form(pX, pY, m, k, n)
        cost, _ = oracle.tree_cost([m, k, n], [pX, pY], [0])
        assert cost == counted
        assert oracle.plan_bruteforce([m, k, n], [pX, pY])["cost"] == counted


def test_result_property_rules():
    n = 6
    want = {(L, L): L, (U, U): U, (L, U): G, (U, L): G, (G, L): G, (L, G): G, (G, U): G, (U, G): G,
            (G, G): G}
    for (a, b), r in want.items():
        assert oracle.tree_cost([n, n, n], [a, b], [0])[1] == r
    # Identity is neutral (A*I = A, I*I = I)
    for a in (G, L, U):
        assert oracle.plan_bruteforce([n, n, n], [a, I])["result_prop"] == a
        assert oracle.plan_bruteforce([n, n, n], [I, a])["result_prop"] == a
    r = oracle.plan_bruteforce([n, n, n], [I, I])
    assert (r["result_prop"], r["cost"], r["n_eff"]) == (I, 0, 0)


def test_paper_listing_5x5_cost_and_property():
    lines = golden_lines("listing_5x5_lower_lower.txt")
    mults = int(lines[1].split()[1])
    r = oracle.plan_bruteforce([5, 5, 5], [L, L])
    assert r["cost"] == mults == oracle.count_mults(5, 5, 5, L, L)
    assert r["result_prop"] == L and lines[0].split()[1] == "lowerTri"


def test_paper_sec4_chain():
    kv = dict(ln.split(" ", 1) for ln in golden_lines("sec4_chain.txt"))
    dims = [int(x) for x in kv["dims"].split()]
    props = [G] * 4
    r = oracle.plan_bruteforce(dims, props)
    assert oracle.plan_string(props, r["splits"]) == kv["chosen"]
    assert r["cost"] == int(kv["chosen_mults"])
    assert r["num_trees"] == 5
    ltr = oracle.left_to_right_splits(props)
    assert oracle.plan_string(props, ltr) == kv["initial"]
    assert oracle.tree_cost(dims, props, ltr)[0] == int(kv["initial_mults"])


def test_workload_optima():
    import synthetic_chains as sc
    for ln in golden_lines("workload_plans.txt"):
        w = ln.split(" ", 5)
        name, cost, plan = w[1], int(w[3]), w[5]
        c = sc.CONFIGS[name]
        r = oracle.plan_bruteforce(c.dims, c.props)
        assert r["cost"] == cost, name
        assert oracle.plan_string(c.props, r["splits"]) == plan, name


def textbook_matrix_chain(dims):
    """Classic O(n^3) matrix-chain-order DP for general matrices."""
    n = len(dims) - 1
    m = [[0] * n for _ in range(n)]
    for length in range(2, n + 1):
        for i in range(n - length + 1):
            j = i + length - 1
            m[i][j] = min(m[i][k] + m[k + 1][j] + dims[i] * dims[k + 1] * dims[j + 1]
                          for k in range(i, j))
    return m[0][n - 1]


def test_general_chains_reduce_to_textbook_dp():
    rng = np.random.default_rng(7)
    for _ in range(300):
        n = int(rng.integers(1, 9))
        dims = [int(x) for x in rng.integers(1, 60, size=n + 1)]
        assert oracle.plan_bruteforce(dims, [G] * n)["cost"] == textbook_matrix_chain(dims)


def test_number_of_trees_is_catalan():
    catalan = [1, 1, 2, 5, 14, 42, 132, 429, 1430]
    for n in range(1, 10):
        assert oracle.plan_bruteforce([3] * (n + 1), [G] * n)["num_trees"] == catalan[n - 1]


def test_bruteforce_minimum_over_python_enumeration():
    # the C enumerator must see the same trees and costs as an enumeration written here
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(1, 7))
        dims, props = random_chain(rng, n, 12)
        surv = oracle.survivors(props)
        r = oracle.plan_bruteforce(dims, props)
        if not surv:
            assert r["cost"] == 0
            continue
        best = None
        for tree in all_preorder_trees(0, len(surv) - 1):
            splits = [surv[s] for s in tree]
            c, _ = oracle.tree_cost(dims, props, splits)
            key = (c, splits)
            if best is None or key < best:
                best = key
        assert (r["cost"], r["splits"]) == best


def test_eliding_identity_equals_zero_cost_identity():
    # dropping Identity factors first, or keeping them at cost 0, gives the same minimum
    rng = np.random.default_rng(13)
    for _ in range(300):
        n = int(rng.integers(1, 8))
        dims, props = random_chain(rng, n, 20)
        a = oracle.plan_bruteforce(dims, props, elide=True)
        b = oracle.plan_bruteforce(dims, props, elide=False)
        assert a["cost"] == b["cost"]
        assert a["result_prop"] == b["result_prop"]


def test_tie_goes_to_smallest_preorder_splits():
    r = oracle.plan_bruteforce([32, 32, 32, 32], [L, G, U])
    assert oracle.tree_cost([32] * 4, [L, G, U], [0, 1])[0] == oracle.tree_cost([32] * 4, [L, G, U], [1, 0])[0]
    assert r["splits"] == [0, 1]
    r = oracle.plan_bruteforce([4] * 6, [G] * 5)       # every tree costs the same
    assert r["splits"] == [0, 1, 2, 3]


def test_malformed_splits_rejected():
    with pytest.raises(ValueError):
        oracle.tree_cost([4, 4, 4, 4], [G, G, G], [2, 0])
    with pytest.raises(ValueError):
        oracle.tree_cost([4, 4, 4, 4], [G, I, G], [1])      # split on an elided factor
