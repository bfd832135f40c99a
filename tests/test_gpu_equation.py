"""GPU parity for sums of chain products (Table 1 "Add", "Mul", "Equation"; Sec. 2
"Operations"): pure variadic Adds of terms with every structure, transposed terms, Identity
terms, and mixed sums of chains, against the oracle's dense definitions."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import D, G, I, L, TOL, U, assert_close_by_tiles, poison_other_half, structure_mask

pytestmark = pytest.mark.gpu


def run_equation(chains, family, flags=0, pad=0):
    """chains: list of (dims, props, trans or None).  Returns (equation, result with NaN sentinel)."""
    host, dev = [], []
    for c, (dims, props, trans) in enumerate(chains):
        h = sc.make_chain(dims, props, family + c, trans=trans)
        host.append(h)
        row = []
        for f, p in zip(h, props):
            if f is None:
                row.append(None)
                continue
            d = poison_other_half(f.cuda(), p)
            if pad:
                wide = torch.full((d.shape[0], d.shape[1] + pad), float("nan"), device="cuda")
                wide[:, :d.shape[1]] = d
                d = wide[:, :d.shape[1]]
            row.append(d)
        dev.append(row)
    eq = mom.mom_equation_plan(chains)
    rows, cols, prop = eq.result
    out_full = torch.full((rows, cols + pad), float("nan"), device="cuda")
    out = out_full[:, :cols]
    ws = torch.full((max(eq.workspace_bytes, 4) // 4,), float("nan"), device="cuda")
    mom.mom_equation_eval(eq, dev, out=out, workspace=ws, flags=flags)
    torch.cuda.synchronize()
    got = out_full.cpu().numpy()
    if pad:
        assert np.all(np.isnan(got[:, cols:]))
    got = got[:, :cols]
    want = oracle.equation_dense([(d, p, [None if f is None else f.numpy() for f in h], t)
                                  for (d, p, t), h in zip(chains, host)])
    assert prop == oracle.equation_property([(d, p, None, t) for d, p, t in chains])
    if prop == I:
        assert np.array_equal(got, np.eye(rows, dtype=np.float32))
        return eq, got
    assert_close_by_tiles(got, want, prop)
    mask = structure_mask(prop, rows, cols)
    if prop in (L, U, D):
        other = got[~mask]
        if flags & mom.MOM_OUT_ZERO_FILL_TRIANGLE:
            assert np.all(other == 0.0)
        else:
            assert np.all(np.isnan(other)), "outside the sum's structure nothing may be written"
    return eq, got


@pytest.mark.parametrize("n", [1, 33, 130, 256])
def test_variadic_add_of_every_structure(n):
    rng = np.random.default_rng(n)
    for trial in range(12):
        k = int(rng.integers(1, 12))                      # more than eight terms take two launches
        props = [int(rng.choice([G, L, U, I, D])) for _ in range(k)]
        if trial % 3 == 0:
            props = [int(rng.choice([L, I, D])) for _ in range(k)]      # sums that stay triangular
        trans = [int(x) for x in rng.integers(0, 2, size=k)]
        chains = [([n, n], [p], [t]) for p, t in zip(props, trans)]
        run_equation(chains, 2700 + trial * 20, flags=int(rng.integers(0, 2)), pad=int(rng.choice([0, 3, 4])))


def test_rectangular_add_with_transposed_terms():
    chains = [([70, 45], [G], None), ([70, 45], [G], [1]), ([70, 45], [G], None)]
    _, got = run_equation(chains, 2900)
    a, b, c = (sc.make_chain(d, p, 2900 + i, trans=t)[0].numpy().astype(np.float64) for i, (d, p, t) in enumerate(chains))
    assert np.max(np.abs(got - (a + b.T + c))) < 1e-5


def test_sums_of_chains_with_products():
    n = 150
    cases = [
        [([n, n, n], [G, G], None), ([n, n], [G], None)],                                  # A B + C
        [([n, n, n], [L, L], None), ([n, n], [I], None), ([n, n, n], [L, L], [0, 0])],     # stays lowerTri
        [([n, n, n], [L, L], None), ([n, n, n], [U, U], None)],                            # L L + U U: no addend fills the sum
        [([n, n, n, n], [L, G, U], None), ([n, n, n], [G, G], [1, 1]), ([n, n], [D], None), ([n, n], [U], [1])],
        [([n, 40, n], [G, G], None), ([n, 2000, n], [G, G], None)],                        # second addend is split along k
        [([n, n, n], [D, D], None), ([n, n], [I], None)],                                  # diagonal sum
    ]
    for i, chains in enumerate(cases):
        for flags in (0, mom.MOM_OUT_ZERO_FILL_TRIANGLE):
            run_equation(chains, 3000 + 10 * i, flags=flags)


def test_large_sum_of_two_products_whole_result():
    n = 2048
    chains = [([n, n, n], [L, G], None), ([n, n, n], [G, U], [1, 0]), ([n, n], [G], None)]
    eq, _ = run_equation(chains, 3100)
    assert eq.workspace_bytes == n * n * 4
