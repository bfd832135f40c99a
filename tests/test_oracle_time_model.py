"""Pins of the oracle's time model and of the brute-force search that minimises it (the opt-in
objective beside the paper's multiplication count; Sec. 2 "Transformations", Sec. 4 "Results")."""
import numpy as np

import oracle
from helpers import all_preorder_trees, golden_lines, random_chain

G, L, U, I = 0, 1, 2, 3


def test_hand_worked_product_times():
    rows = [[int(x) for x in ln.split()] for ln in golden_lines("time_model.txt")]
    assert len(rows) >= 9
    for m, k, n, px, py, want in rows:
        assert oracle.product_time_ps(m, k, n, px, py) == want, (m, k, n, px, py)


def test_large_whole_tile_general_products_cost_their_flop_at_the_peak():
    # m, n multiples of 128 with more than 256 tiles, k a multiple of 32 and matrix-bound:
    # time - launch = m*n*k*2 FLOP at 256 compute units * 256 FLOP per clock * 2.4 GHz, up to the
    # rounding of the chunk constant and of ceil(chunks / 256)
    for m, k, n in ((4096, 4096, 4096), (2048, 8192, 4096), (8192, 1024, 2048)):
        t = oracle.product_time_ps(m, k, n, G, G) - 6000000
        ideal = 2.0 * m * k * n / 157.2864e12 * 1e12
        assert abs(t - ideal) / ideal < 1e-3


def test_triangular_products_cost_about_half():
    n = 4096
    full = oracle.product_time_ps(n, n, n, G, G) - 6000000
    tri = oracle.product_time_ps(n, n, n, L, G) - 6000000
    assert 0.5 < tri / full < 0.53            # (nt + 1) / (2 nt) with nt = 32 tile rows
    assert oracle.product_time_ps(n, n, n, U, G) == oracle.product_time_ps(n, n, n, L, G)
    assert oracle.product_time_ps(n, n, n, G, L) == oracle.product_time_ps(n, n, n, G, U)
    assert oracle.product_time_ps(n, n, n, L, L) == oracle.product_time_ps(n, n, n, U, U)
    assert oracle.product_time_ps(n, n, n, L, U) == oracle.product_time_ps(n, n, n, U, L)
    assert oracle.product_time_ps(n, n, n, L, L) < oracle.product_time_ps(n, n, n, L, U) < tri + 6000000
    assert oracle.product_time_ps(n, n, n, I, G) == 0


def test_time_grows_with_every_dimension():
    rng = np.random.default_rng(3)
    for _ in range(300):
        m, k, n = (int(x) for x in rng.integers(1, 700, size=3))
        t = oracle.product_time_ps(m, k, n, G, G)
        assert t >= 6000000
        # (k may cross the threshold at which the product is cut into slices, which is allowed to pay)
        assert oracle.product_time_ps(m + 128, k, n, G, G) >= t or m <= 64 < m + 128
        assert oracle.product_time_ps(m, k, n + 128, G, G) >= t or n <= 64 < n + 128


def python_best_tree(dims, props):
    """Independent enumeration in Python: every tree, cost = sum of product_time_ps."""
    surv = [i for i, p in enumerate(props) if p != I]
    d = [dims[i] for i in surv] + [dims[-1]]
    p = [props[i] for i in surv]

    def join(a, b):
        return a if a == b and a in (L, U) else G

    def walk(lo, hi, it):
        if lo == hi:
            return d[lo], d[lo + 1], p[lo], 0
        s = next(it)
        ar, ac, ap, at = walk(lo, s, it)
        br, bc, bp, bt = walk(s + 1, hi, it)
        return ar, bc, join(ap, bp), at + bt + oracle.product_time_ps(ar, ac, bc, ap, bp)

    best = None
    for tree in all_preorder_trees(0, len(surv) - 1):
        cost = walk(0, len(surv) - 1, iter(tree))[3]
        if best is None or (cost, tree) < best:
            best = (cost, tree)
    return best[0], [surv[s] for s in best[1]]


def test_bruteforce_time_equals_python_enumeration():
    rng = np.random.default_rng(4)
    pool = [1, 7, 33, 64, 65, 96, 130, 256, 300, 1000, 2050]
    for trial in range(150):
        n = int(rng.integers(1, 7))
        props = [int(rng.choice([G, G, L, U, I])) for _ in range(n)]
        dims = [int(rng.choice(pool))]
        for q in props:
            dims.append(dims[-1] if q != G else int(rng.choice(pool)))
        if all(q == I for q in props):
            continue
        got = oracle.plan_bruteforce_time(dims, props)
        cost, splits = python_best_tree(dims, props)
        assert (got["time_ps"], got["splits"]) == (cost, splits)
        assert got["mults"] == oracle.tree_cost(dims, props, got["splits"])[0]
        assert oracle.tree_time_ps(dims, props, got["splits"]) == cost


def test_large_matrix_bound_general_chains_get_the_multiplication_optimal_tree():
    # the Sec. 4 chain scaled to multiples of 128 with every product matrix-bound on many tiles:
    # the time model then orders trees as the multiplication count does
    dims = [x * 128 for x in (8, 11, 9, 12, 4)]
    a, b = oracle.plan_bruteforce(dims, [G] * 4), oracle.plan_bruteforce_time(dims, [G] * 4)
    assert a["splits"] == b["splits"] and a["cost"] == b["mults"]


def test_a_chain_where_the_two_objectives_part():
    # general * general * general * lowerTri, 256 x 1024 x 4096 x 256 x 256: the fewest multiplications
    # are in ((0 (1 2)) 3), three dependent products of which the first has few tiles and a long k;
    # the time model prefers ((0 1) (2 3)): 1.29 times as many, in two independent products and a root
    dims, props = [256, 1024, 4096, 256, 256], [G, G, G, L]
    a, b = oracle.plan_bruteforce(dims, props), oracle.plan_bruteforce_time(dims, props)
    assert a["splits"] == [2, 0, 1] and b["splits"] == [1, 0, 2]
    assert b["mults"] > 1.25 * a["cost"]
    assert oracle.tree_time_ps(dims, props, a["splits"]) > 1.1 * b["time_ps"]
