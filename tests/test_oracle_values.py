"""Pins for the oracle's value side: dense definition, row sampling, tree evaluation."""
import numpy as np
import pytest

import oracle
import synthetic_chains as sc
from helpers import all_preorder_trees, golden_lines, random_chain

G, L, U, I = 0, 1, 2, 3


def np_factors(dims, props, family):
    return [None if f is None else f.numpy() for f in sc.make_chain(dims, props, family)]


def dense64(f, n):
    return np.eye(n) if f is None else f.astype(np.float64)


def test_paper_listing_5x5_values():
    lines = golden_lines("listing_5x5_lower_lower.txt")
    want = np.array([[float(x) for x in ln.split()] for ln in lines[2:]])
    a = np.tril(np.ones((5, 5), dtype=np.float32))
    got = oracle.eval_dense([5, 5, 5], [L, L], [a, a])
    assert np.array_equal(got, want)
    got2, prop = oracle.eval_plan([5, 5, 5], [L, L], [a, a], [0])
    assert prop == L and np.array_equal(got2, want)
    assert np.array_equal(oracle.eval_rows([5, 5, 5], [L, L], [a, a], [4, 0]), want[[4, 0]])


def test_dense_matches_numpy_matmul_f64():
    # rectangular, all different dims: a transposed operand or swapped index cannot pass
    dims = [7, 13, 5, 11, 3]
    props = [G] * 4
    f = np_factors(dims, props, 91)
    want = np.linalg.multi_dot([x.astype(np.float64) for x in f])
    got = oracle.eval_dense(dims, props, f)
    assert np.allclose(got, want, rtol=1e-13, atol=1e-13)
    rows = [6, 0, 3]
    assert np.allclose(oracle.eval_rows(dims, props, f, rows), want[rows], rtol=1e-13, atol=1e-13)


def test_identity_rules_bit_exact():
    a = sc.make_factor(9, 9, G, 5).numpy()
    for dims, props, fac in (([9, 9, 9], [G, I], [a, None]), ([9, 9, 9], [I, G], [None, a]),
                             ([9, 9, 9, 9], [I, G, I], [None, a, None])):
        assert np.array_equal(oracle.eval_dense(dims, props, fac), a.astype(np.float64))
        assert np.array_equal(oracle.eval_plan(dims, props, fac, [])[0], a.astype(np.float64))
        assert np.array_equal(oracle.eval_rows(dims, props, fac, [2, 8]), a.astype(np.float64)[[2, 8]])
    eye = np.eye(6)
    assert np.array_equal(oracle.eval_dense([6, 6, 6], [I, I], [None, None]), eye)
    out, prop = oracle.eval_plan([6, 6, 6], [I, I], [None, None], [])
    assert prop == I and np.array_equal(out, eye)


@pytest.mark.parametrize("pa,pb,keeps", [(L, L, L), (U, U, U), (L, U, G), (U, L, G)])
def test_structure_invariants(pa, pb, keeps):
    n = 17
    f = np_factors([n, n, n], [pa, pb], 33)
    c = oracle.eval_dense([n, n, n], [pa, pb], f)
    if keeps == L:
        assert np.all(np.triu(c, 1) == 0.0)
    elif keeps == U:
        assert np.all(np.tril(c, -1) == 0.0)
    else:
        assert np.count_nonzero(np.triu(c, 1)) > 0 and np.count_nonzero(np.tril(c, -1)) > 0
    assert oracle.eval_plan([n, n, n], [pa, pb], f, [0])[1] == keeps


def test_every_tree_agrees_with_dense_definition():
    rng = np.random.default_rng(3)
    for trial in range(40):
        n = int(rng.integers(1, 6))
        dims, props = random_chain(rng, n, 9)
        f = np_factors(dims, props, 200 + trial)
        want = oracle.eval_dense(dims, props, f)
        scale = max(np.linalg.norm(want), 1e-300)
        surv = oracle.survivors(props)
        trees = list(all_preorder_trees(0, len(surv) - 1)) if surv else [[]]
        for tree in trees:
            got, _ = oracle.eval_plan(dims, props, f, [surv[s] for s in tree])
            assert np.linalg.norm(got - want) / scale <= 1e-12


def test_tree_evaluation_ignores_the_other_half():
    # triangular factors are defined by their triangle: garbage in the other half of the
    # buffer must not reach a tree evaluation, which reads only the structure
    n = 8
    f = np_factors([n, n, n, 5], [L, U, G], 44)
    want, _ = oracle.eval_plan([n, n, n, 5], [L, U, G], f, [0, 1])
    dirty = [f[0] + np.triu(np.full((n, n), 7.0, np.float32), 1),
             f[1] + np.tril(np.full((n, n), -3.0, np.float32), -1), f[2]]
    got, _ = oracle.eval_plan([n, n, n, 5], [L, U, G], dirty, [0, 1])
    assert np.array_equal(got, want)


def test_rows_match_dense_on_mixed_chain():
    dims, props = [12, 12, 12, 12, 12, 7], [L, I, L, U, G]
    f = np_factors(dims, props, 77)
    full = oracle.eval_dense(dims, props, f)
    rows = [11, 0, 5]
    assert np.allclose(oracle.eval_rows(dims, props, f, rows), full[rows], rtol=1e-13, atol=1e-14)
    want = np.linalg.multi_dot([dense64(x, 12) for x in f])
    assert np.allclose(full, want, rtol=1e-12, atol=1e-13)


def test_generator_enforces_property_zeros():
    a = sc.make_factor(10, 10, L, 1).numpy()
    b = sc.make_factor(10, 10, U, 1).numpy()
    assert np.all(np.triu(a, 1) == 0) and np.all(np.tril(b, -1) == 0)
    assert np.all(np.abs(a) <= 1) and np.count_nonzero(np.diag(a)) == 10
    assert sc.make_factor(10, 10, I, 1) is None
    again = sc.make_factor(10, 10, L, 1).numpy()
    assert np.array_equal(a, again)
