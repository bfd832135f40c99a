"""Pins of the diagonal property, the set {lowerTri, upperTri} (Sec. 2 "Matrix Attribute": a
matrix carries a set of non-conflicting properties): counted multiplications, structure of
products, values against numpy's row / column scaling."""
import numpy as np

import oracle
import synthetic_chains as sc
from helpers import all_preorder_trees

G, L, U, I, D = 0, 1, 2, 3, 4


def pattern(prop, rows, cols):
    ones = np.ones((rows, cols), dtype=np.int64)
    return {G: ones, L: np.tril(ones), U: np.triu(ones), D: np.tril(np.triu(ones)), I: np.eye(rows, cols, dtype=np.int64)}[prop]


def rel(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def test_counted_multiplications_and_closed_forms_with_a_diagonal_operand():
    for px in (G, L, U, D):
        for py in (G, L, U, D):
            if D not in (px, py):
                continue
            for n in range(1, 10):
                m = n if px != G else n + 2
                c = n if py != G else n + 3
                counted = oracle.count_mults(m, n, c, px, py)
                assert counted == int((pattern(px, m, n) @ pattern(py, n, c)).sum())
                assert oracle.tree_cost([m, n, c], [px, py], [0])[0] == counted
    assert oracle.tree_cost([7, 7, 7], [D, D], [0]) == (7, D)
    assert oracle.tree_cost([7, 7, 7], [D, L], [0]) == (28, L)
    assert oracle.tree_cost([7, 7, 7], [U, D], [0]) == (28, U)
    assert oracle.tree_cost([7, 7, 3], [D, G], [0]) == (21, G)
    assert oracle.tree_cost([7, 7, 7], [D, I], []) == (0, D)
    assert oracle.transposed_property(D) == D


def test_diagonal_products_are_row_and_column_scalings():
    n = 9
    d = sc.make_factor(n, n, D, 1).numpy()
    assert np.count_nonzero(d - np.diag(np.diag(d))) == 0
    a = sc.make_factor(n, 6, G, 2).numpy()
    b = sc.make_factor(5, n, G, 3).numpy()
    dv = np.diag(d).astype(np.float64)
    got = oracle.eval_dense([n, n, 6], [D, G], [d, a])
    assert rel(got, dv[:, None] * a.astype(np.float64)) < 1e-15
    got, prop = oracle.eval_plan([5, n, n], [G, D], [b, d], [0])
    assert prop == G and rel(got, b.astype(np.float64) * dv[None, :]) < 1e-15
    lo = sc.make_factor(n, n, L, 4).numpy()
    got, prop = oracle.eval_plan([n, n, n], [D, L], [d, lo], [0])
    assert prop == L and np.all(np.triu(got, 1) == 0) and rel(got, dv[:, None] * lo.astype(np.float64)) < 1e-15
    got, prop = oracle.eval_plan([n, n, n], [D, D], [d, d], [0])
    assert prop == D and rel(got, np.diag(dv * dv)) < 1e-15


def test_tree_evaluation_reads_only_the_diagonal():
    n = 8
    dims, props = [n, n, n, 5], [D, U, G]
    f = [x.numpy().copy() for x in sc.make_chain(dims, props, 31)]
    want = oracle.eval_dense(dims, props, f)
    f[0][~np.eye(n, dtype=bool)] = 1e30
    for splits in ([0, 1], [1, 0]):
        got, _ = oracle.eval_plan(dims, props, f, splits)
        assert rel(got, want) < 1e-13


def test_every_tree_with_diagonal_factors_agrees_with_dense():
    rng = np.random.default_rng(17)
    for trial in range(40):
        n = int(rng.integers(2, 6))
        props = [int(rng.choice([G, L, U, D, D, I])) for _ in range(n)]
        dims = [int(rng.integers(1, 12))]
        for p in props:
            dims.append(dims[-1] if p != G else int(rng.integers(1, 12)))
        f = [None if x is None else x.numpy() for x in sc.make_chain(dims, props, 500 + trial)]
        want = oracle.eval_dense(dims, props, f)
        surv = oracle.survivors(props)
        if not surv:
            continue
        best = oracle.plan_bruteforce(dims, props)
        costs = []
        for tree in all_preorder_trees(0, len(surv) - 1):
            splits = [surv[s] for s in tree]
            got, prop = oracle.eval_plan(dims, props, f, splits)
            assert rel(got, want) < 1e-12 or np.linalg.norm(want) == 0
            costs.append(oracle.tree_cost(dims, props, splits)[0])
            assert prop == best["result_prop"]
        assert min(costs) == best["cost"]


def test_time_model_of_a_scaling_pass_is_memory_only():
    n = 4096
    assert oracle.product_time_ps(n, n, n, D, G) == 6000000 + 4 * (n + 2 * n * n) // 8
    assert oracle.product_time_ps(n, n, n, L, D) == 6000000 + 4 * (n + n * (n + 1)) // 8
    assert oracle.product_time_ps(n, n, n, D, D) == 6000000 + 4 * 3 * n // 8
