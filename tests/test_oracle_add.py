"""Pins of the oracle's variadic Add and of sums of chains (Table 1 "Add"; Sec. 2 "Operations")."""
import itertools

import numpy as np

import oracle
import synthetic_chains as sc

G, L, U, I, D = 0, 1, 2, 3, 4


def pattern(prop, n):
    ones = np.ones((n, n), dtype=bool)
    return {G: ones, L: np.tril(ones), U: np.triu(ones), D: np.eye(n, dtype=bool), I: np.eye(n, dtype=bool)}[prop]


def test_sum_property_is_the_smallest_structure_that_holds_every_term():
    n = 4
    order = [D, L, U, G]            # candidates for a sum of two or more terms, small to large (L, U incomparable)
    for k in (2, 3):
        for props in itertools.product([G, L, U, I, D], repeat=k):
            union = np.zeros((n, n), dtype=bool)
            for p in props:
                union |= pattern(p, n)
            got = oracle.sum_property(list(props))
            assert got != I
            assert not np.any(union & ~pattern(got, n))                         # holds every term
            for smaller in order:
                if pattern(smaller, n).sum() < pattern(got, n).sum():
                    assert np.any(union & ~pattern(smaller, n))                 # and nothing smaller does
    for p in (G, L, U, I, D):
        assert oracle.sum_property([p]) == p
    assert oracle.sum_property([L, L], trans=[1, 0]) == G and oracle.sum_property([L, U], trans=[1, 0]) == U


def test_add_against_numpy_with_transposed_terms():
    rng = np.random.default_rng(1)
    rows, cols = 7, 5
    for trial in range(10):
        k = int(rng.integers(1, 6))
        trans = [int(x) for x in rng.integers(0, 2, size=k)]
        terms = [rng.uniform(-1, 1, (cols, rows) if t else (rows, cols)).astype(np.float32) for t in trans]
        want = sum((x.T if t else x).astype(np.float64) for x, t in zip(terms, trans))
        got = oracle.add_dense(rows, cols, [G] * k, terms, trans=trans)
        assert np.max(np.abs(got - want)) < 1e-14


def test_add_structures_and_identity_terms():
    n = 6
    lo = [sc.make_factor(n, n, L, s).numpy() for s in (1, 2)]
    got = oracle.add_dense(n, n, [L, L], lo)
    assert np.all(np.triu(got, 1) == 0) and np.array_equal(got, lo[0].astype(np.float64) + lo[1].astype(np.float64))
    assert np.array_equal(oracle.add_dense(n, n, [I, I], [None, None]), 2 * np.eye(n))
    g = sc.make_factor(n, n, G, 3).numpy()
    assert np.array_equal(oracle.add_dense(n, n, [G], [g]), g.astype(np.float64))            # one term: the term
    assert np.array_equal(oracle.add_dense(n, n, [G, I], [g, None]), g.astype(np.float64) + np.eye(n))
    sym = oracle.add_dense(n, n, [G, G], [g, g], trans=[0, 1])                               # X + X^T
    assert np.array_equal(sym, sym.T)


def test_sum_of_chains_against_numpy():
    rng = np.random.default_rng(2)
    a = rng.uniform(-1, 1, (6, 9)).astype(np.float32)
    b = rng.uniform(-1, 1, (9, 4)).astype(np.float32)
    c = rng.uniform(-1, 1, (6, 4)).astype(np.float32)
    d = rng.uniform(-1, 1, (4, 6)).astype(np.float32)
    chains = [([6, 9, 4], [G, G], [a, b], None), ([6, 4], [G], [c], None), ([6, 4], [G], [d], [1])]
    want = a.astype(np.float64) @ b.astype(np.float64) + c + d.T.astype(np.float64)
    assert np.max(np.abs(oracle.equation_dense(chains) - want)) < 1e-13
    assert oracle.equation_property(chains) == G
    lo = sc.make_factor(5, 5, L, 4).numpy()
    chains = [([5, 5, 5], [L, L], [lo, lo], None), ([5, 5], [I], [None], None)]
    assert oracle.equation_property(chains) == L
