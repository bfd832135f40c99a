"""GPU parity for factors that enter the chain transposed (Table 1 "Transpose"; Sec. 2
"Transformations": lowerTri(A) -> upperTri(A^T)): the product kernels read the stored buffer
as it is, so every property pair is checked in all four combinations of transposed operands,
element by element against the dense f64 oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, I, L, TOL, U, assert_close_by_tiles, check_against_dense, eval_chain, rel_fro, upload
from helpers import all_preorder_trees, random_chain

pytestmark = pytest.mark.gpu

PAIRS = [(a, b) for a in (G, L, U) for b in (G, L, U)]
COMBOS = [(0, 0), (1, 0), (0, 1), (1, 1)]


@pytest.mark.parametrize("ta,tb", COMBOS)
@pytest.mark.parametrize("n", [33, 130, 300])
def test_every_property_pair_transposed_ragged(ta, tb, n):
    # several tiles plus a ragged tail, unaligned rows: loads 4 bytes wide through the bounded descriptors
    for pa, pb in PAIRS:
        m = n if pa != G else n + 7
        c = n if pb != G else max(n - 5, 1)
        dims, props, trans = [m, n, c], [pa, pb], [ta, tb]
        check_against_dense(dims, props, sc.make_chain(dims, props, 1300 + n, trans=trans), trans=trans)


@pytest.mark.parametrize("ta,tb", COMBOS)
@pytest.mark.parametrize("n", [128, 384, 640])
def test_every_property_pair_transposed_whole_tiles(ta, tb, n):
    # nothing ragged: 16-byte loads, steady-state chunk body, diagonals masked at staging
    for pa, pb in PAIRS:
        dims, props, trans = [n, n, n], [pa, pb], [ta, tb]
        check_against_dense(dims, props, sc.make_chain(dims, props, 1400 + n, trans=trans), trans=trans)


@pytest.mark.parametrize("ta,tb", COMBOS[1:])
def test_transposed_rectangular_and_short_side_products(ta, tb):
    # 64x64 tile shape (a side <= 64), split-K, and rectangular general operands
    for m, k, n in ((64, 1000, 64), (500, 40, 700), (33, 4097, 17), (512, 8192, 64), (200, 96, 48), (1, 1, 1)):
        dims, props, trans = [m, k, n], [G, G], [ta, tb]
        check_against_dense(dims, props, sc.make_chain(dims, props, 1500 + m, trans=trans), trans=trans)


def test_transposed_strided_buffers_and_zero_fill():
    n = 200
    for pa, pb, trans in ((L, L, [1, 1]), (L, U, [1, 0]), (U, G, [1, 0]), (G, L, [0, 1])):
        dims, props = [n, n, n], [pa, pb]
        check_against_dense(dims, props, sc.make_chain(dims, props, 1600, trans=trans), trans=trans,
                            flags=mom.MOM_OUT_ZERO_FILL_TRIANGLE, pad_cols=12, out_pad=20)
        check_against_dense(dims, props, sc.make_chain(dims, props, 1601, trans=trans), trans=trans, pad_cols=3, out_pad=1)


def test_random_chains_with_transposed_factors_every_tree():
    rng = np.random.default_rng(31)
    for trial in range(30):
        n = int(rng.integers(1, 6))
        dims, props = random_chain(rng, n, int(rng.choice([60, 200])))
        trans = [int(x) for x in rng.integers(0, 2, size=n)]
        f = sc.make_chain(dims, props, 1700 + trial, trans=trans)
        plan, _ = check_against_dense(dims, props, f, trans=trans, flags=int(rng.integers(0, 2)))
        want = oracle.plan_bruteforce(dims, props, trans=trans)
        assert (plan.cost_mults, plan.splits) == (want["cost"], want["splits"])
        surv = oracle.survivors(props)
        if 3 <= len(surv) <= 4:
            for tree in all_preorder_trees(0, len(surv) - 1):
                check_against_dense(dims, props, f, splits=[surv[s] for s in tree], trans=trans)


def test_single_transposed_factor_is_a_transposing_copy():
    a = sc.make_factor(70, 45, G, 9)
    plan, got = eval_chain([45, 70, 70], [G, I], [a, None], trans=[1, 0])
    assert mom.mom_plan_num_products(plan) == 0 and plan.result == (45, 70, G)
    assert np.array_equal(got, a.numpy().T)
    lo = sc.make_factor(70, 70, L, 10)
    plan, got = eval_chain([70, 70], [L], [lo], trans=[1])
    assert plan.result == (70, 70, U)
    up = np.triu(np.ones((70, 70), dtype=bool))
    assert np.array_equal(got[up], lo.numpy().T[up]) and np.all(np.isnan(got[~up]))


@pytest.mark.parametrize("rows,cols", [(256, 192), (300, 452), (64, 64)])
def test_transposing_copy_whole_blocks_and_edges(rows, cols):
    # blocks of 64 x 64 that lie wholly inside move 16 bytes at a time, the rest element by element;
    # a strided output keeps its padding
    a = sc.make_factor(rows, cols, G, 12)
    for pad in (0, 4, 5):
        plan, got = eval_chain([cols, rows], [G], [a], trans=[1], pad_cols=pad, out_pad=pad)
        assert plan.result == (cols, rows, G) and np.array_equal(got, a.numpy().T)
    if rows == cols or rows == 256:
        n = rows
        for prop, keep in ((L, np.triu), (U, np.tril)):
            t = sc.make_factor(n, n, prop, 13)
            plan, got = eval_chain([n, n], [prop], [t], trans=[1])
            mask = keep(np.ones((n, n), dtype=bool))
            assert np.array_equal(got[mask], t.numpy().T[mask]) and np.all(np.isnan(got[~mask]))


def test_gram_matrix_is_symmetric_bit_for_bit_or_close():
    x = sc.make_factor(300, 200, G, 11)
    _, got = eval_chain([300, 200, 300], [G, G], [x, x], trans=[0, 1])       # X * X^T
    want = x.numpy().astype(np.float64) @ x.numpy().astype(np.float64).T
    assert rel_fro(got, want) <= TOL
    assert rel_fro(got, got.T) <= TOL


def test_batched_chains_with_transposed_factors():
    batch = 37
    for dims, props, trans in (([32, 32, 32, 32], [L, G, U], [1, 0, 1]), ([32, 32, 32, 32], [L, G, U], [0, 1, 0]),
                               ([20, 32, 7, 32], [G, G, G], [1, 1, 0]), ([32, 32], [U], [1])):
        host = sc.make_chain(dims, props, 1800, batch=batch, trans=trans)
        plan = mom.mom_chain_plan(dims, props, trans=trans)
        out = mom.mom_chain_eval_batched(plan, [f.cuda() for f in host])
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        for b in range(batch):
            want = oracle.eval_dense(dims, props, [f[b].numpy() for f in host], trans=trans)
            assert rel_fro(got[b], want) <= TOL


@pytest.mark.parametrize("trans", [[1, 0], [0, 1], [1, 1]])
def test_transposed_trmm4096_whole_result(trans):
    # the single-product workload with its operands stored transposed: U^T * G, L * G^T, U^T * G^T
    n = 4096
    dims, props = [n, n, n], [U if trans[0] else L, G]
    host = sc.make_chain(dims, props, 1900, trans=trans)
    plan = mom.mom_chain_plan(dims, props, trans=trans)
    assert plan.result == (n, n, G) and plan.cost_mults == n * n * (n + 1) // 2
    dev = upload(host, props, poison=True)
    out = torch.full((n, n), float("nan"), device="cuda")
    mom.mom_chain_eval(plan, dev, out=out)
    torch.cuda.synchronize()
    want, _ = oracle.eval_plan(dims, props, [f.numpy() for f in host], plan.splits, trans=trans)
    assert_close_by_tiles(out.cpu().numpy(), want, G)


LARGE_TILE_CASES = [
    ([1801, 1803, 1799], [G, G]),     # 15 x 15 tiles of 128, nothing aligned: every load 4 bytes wide
    ([2899, 2899, 2899], [L, G]),     # one triangle, 23 x 23 tiles, unaligned
    ([2900, 2900, 2900], [G, U]),     # the same from the right, rows 16-byte aligned, ragged last tiles
    ([4868, 4868, 4868], [L, L]),     # two triangles, 39 tile rows: a triangular or a general result
]


@pytest.mark.parametrize("ta,tb", COMBOS)
@pytest.mark.parametrize("dims,props", LARGE_TILE_CASES)
def test_large_tiles_in_every_orientation_ragged_and_unaligned(dims, props, ta, tb):
    # sizes at which the 128 x 128 tile shape is chosen (the small cases above all run on 64 x 64 tiles):
    # edges, diagonals and 4-byte loads of all four kernel orientations, whole results
    trans = [ta, tb]
    host = sc.make_chain(dims, props, 1950, trans=trans)
    plan = mom.mom_chain_plan(dims, props, trans=trans)
    rows, cols, prop = plan.result
    dev = upload(host, props, poison=True)
    out = torch.full((rows, cols), float("nan"), device="cuda")
    mom.mom_chain_eval(plan, dev, out=out)
    torch.cuda.synchronize()
    want, want_prop = oracle.eval_plan(dims, props, [f.numpy() for f in host], plan.splits, trans=trans)
    assert want_prop == prop
    assert_close_by_tiles(out.cpu().numpy(), want, prop)
