"""Pins of the oracle's transposed factors (Table 1 "Transpose"; Sec. 2 "Transformations": the
transpose of a lowerTri matrix is upperTri) against numpy and against the oracle's own
untransposed functions on explicitly transposed copies."""
import numpy as np
import pytest

import oracle
import synthetic_chains as sc
from helpers import all_preorder_trees, random_chain

G, L, U, I = 0, 1, 2, 3


def np_chain(dims, props, trans, factors):
    """The chain by numpy in f64: stored matrices transposed where flagged, eye for Identity."""
    mats = []
    for t, (p, f) in enumerate(zip(props, factors)):
        if p == I:
            mats.append(np.eye(dims[t]))
        else:
            a = f.astype(np.float64)
            mats.append(a.T if trans[t] else a)
    out = mats[0]
    for m in mats[1:]:
        out = out @ m
    return out


def rel(a, b):
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def test_transposed_property_rule():
    assert [oracle.transposed_property(p) for p in (G, L, U, I)] == [G, U, L, I]
    assert oracle.chain_props([L, U, G, I, L], [1, 1, 1, 1, 0]) == [U, L, G, I, L]
    # mirrored pattern, entry by entry: (i,j) is structural in A^T iff (j,i) is in A
    for p in (G, L, U):
        q = oracle.transposed_property(p)
        for i in range(4):
            for j in range(4):
                in_a = (j <= i) if p == L else (j >= i) if p == U else True
                in_at = (i <= j) if q == L else (i >= j) if q == U else True
                # A^T[j][i] = A[i][j]
                assert in_a == in_at


def test_product_transposed_equals_reversed_product_of_transposes():
    # (A B)^T = B^T A^T, all dimensions different
    rng = np.random.default_rng(5)
    a = rng.uniform(-1, 1, (7, 11)).astype(np.float32)
    b = rng.uniform(-1, 1, (11, 5)).astype(np.float32)
    want = (a.astype(np.float64) @ b.astype(np.float64)).T
    got = oracle.eval_dense([5, 11, 7], [G, G], [b, a], trans=[1, 1])
    assert rel(got, want) < 1e-14
    # one side only: A^T stored as a, times a matching right factor
    c = rng.uniform(-1, 1, (7, 3)).astype(np.float32)
    got = oracle.eval_dense([11, 7, 3], [G, G], [a, c], trans=[1, 0])
    assert rel(got, a.astype(np.float64).T @ c.astype(np.float64)) < 1e-14
    d = rng.uniform(-1, 1, (3, 11)).astype(np.float32)
    got = oracle.eval_dense([7, 11, 3], [G, G], [a, d], trans=[0, 1])
    assert rel(got, a.astype(np.float64) @ d.astype(np.float64).T) < 1e-14


def test_dense_with_transposes_against_numpy_on_rectangular_chains():
    rng = np.random.default_rng(6)
    dims = [6, 9, 4, 13, 5, 8]
    for trial in range(16):
        trans = [int(x) for x in rng.integers(0, 2, size=5)]
        props = [G] * 5
        f = [rng.uniform(-1, 1, (dims[t + 1], dims[t]) if trans[t] else (dims[t], dims[t + 1])).astype(np.float32)
             for t in range(5)]
        want = np_chain(dims, props, trans, f)
        assert rel(oracle.eval_dense(dims, props, f, trans=trans), want) < 1e-13
        rows = [0, 3, 5]
        assert rel(oracle.eval_rows(dims, props, f, rows, trans=trans), want[rows]) < 1e-13
        want2 = np.linalg.multi_dot([(x.T if t else x).astype(np.float64) for x, t in zip(f, trans)])
        assert rel(oracle.eval_dense(dims, props, f, trans=trans), want2) < 1e-13


def test_transposed_lower_is_upper_and_products_keep_their_triangle():
    n = 9
    lo = sc.make_factor(n, n, L, 1).numpy()
    up = sc.make_factor(n, n, U, 2).numpy()
    # L^T * U: both upperTri inside the chain -> the strict lower half of the dense result is exactly 0
    got = oracle.eval_dense([n, n, n], [L, U], [lo, up], trans=[1, 0])
    assert np.all(np.tril(got, -1) == 0.0) and np.any(np.triu(got) != 0.0)
    assert oracle.plan_bruteforce([n, n, n], [L, U], trans=[1, 0])["result_prop"] == U
    # L * U^T: lowerTri * lowerTri
    got = oracle.eval_dense([n, n, n], [L, U], [lo, up], trans=[0, 1])
    assert np.all(np.triu(got, 1) == 0.0)
    assert oracle.plan_bruteforce([n, n, n], [L, U], trans=[0, 1])["result_prop"] == L
    # L^T * L: upper * lower -> general
    assert oracle.plan_bruteforce([n, n, n], [L, L], trans=[1, 0])["result_prop"] == G


def test_costs_and_plans_are_those_of_the_mirrored_chain():
    # cost of L^T * G equals that of U * G, counted one by one on the mirrored pattern
    for n, c in ((1, 1), (5, 3), (8, 8)):
        cost, prop = oracle.tree_cost([n, n, c], [L, G], [0], trans=[1, 0])
        assert (cost, prop) == (oracle.count_mults(n, n, c, U, G), G)
        cost, prop = oracle.tree_cost([c, n, n], [G, U], [0], trans=[0, 1])
        assert (cost, prop) == (oracle.count_mults(c, n, n, G, L), G)
        cost, prop = oracle.tree_cost([n, n, n], [L, U], [0], trans=[1, 0])
        assert (cost, prop) == (oracle.count_mults(n, n, n, U, U), U)
    rng = np.random.default_rng(8)
    for trial in range(300):
        n = int(rng.integers(1, 8))
        dims, props = random_chain(rng, n, 30)
        trans = [int(x) for x in rng.integers(0, 2, size=n)]
        a = oracle.plan_bruteforce(dims, props, trans=trans)
        b = oracle.plan_bruteforce(dims, oracle.chain_props(props, trans))
        assert a == b


def test_every_tree_with_transposed_factors_agrees_with_dense_definition():
    rng = np.random.default_rng(9)
    for trial in range(30):
        n = int(rng.integers(2, 6))
        dims, props = random_chain(rng, n, 14)
        trans = [int(x) for x in rng.integers(0, 2, size=n)]
        f = [None if x is None else x.numpy() for x in sc.make_chain(dims, props, 400 + trial, trans=trans)]
        want = oracle.eval_dense(dims, props, f, trans=trans)
        assert rel(want, np_chain(dims, props, trans, f)) < 1e-13
        surv = oracle.survivors(props)
        for tree in all_preorder_trees(0, max(len(surv) - 1, 0)):
            splits = [surv[s] for s in tree]
            got, rprop = oracle.eval_plan(dims, props, f, splits, trans=trans)
            assert rel(got, want) < 1e-12 or np.linalg.norm(want) == 0
            assert rprop == oracle.tree_cost(dims, props, splits, trans=trans)[1]


def test_tree_evaluation_ignores_the_zero_half_of_a_transposed_triangle():
    n = 12
    dims, props, trans = [n, n, n, 7], [L, U, G], [1, 1, 0]
    f = [x.numpy().copy() for x in sc.make_chain(dims, props, 77, trans=trans)]
    want = oracle.eval_dense(dims, props, f, trans=trans)
    f[0][np.triu_indices(n, 1)] = 1e30        # garbage above the diagonal of the STORED lowerTri
    f[1][np.tril_indices(n, -1)] = -1e30      # garbage below the diagonal of the STORED upperTri
    for splits in ([0, 1], [1, 0]):
        got, _ = oracle.eval_plan(dims, props, f, splits, trans=trans)
        assert rel(got, want) < 1e-12


def test_gram_matrix_is_symmetric():
    x = sc.make_factor(10, 6, G, 3).numpy()
    got = oracle.eval_dense([10, 6, 10], [G, G], [x, x], trans=[0, 1])      # X * X^T
    assert np.array_equal(got, got.T)
    assert rel(got, x.astype(np.float64) @ x.astype(np.float64).T) < 1e-14


def test_untransposed_calls_are_unchanged():
    dims, props = [5, 5, 8, 3], [L, G, G]
    f = [x.numpy() for x in sc.make_chain(dims, props, 12)]
    a = oracle.eval_dense(dims, props, f)
    b = oracle.eval_dense(dims, props, f, trans=[0, 0, 0])
    assert np.array_equal(a, b)
    c, _ = oracle.eval_plan(dims, props, f, [1, 0])
    d, _ = oracle.eval_plan(dims, props, f, [1, 0], trans=[0, 0, 0])
    assert np.array_equal(c, d)
