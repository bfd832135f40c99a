"""GPU parity of WHOLE results at the sizes where the large-launch paths of the product kernel
run: tiles paired longest-with-shortest, the persistent grid over equal tiles, and tile orders
that take many rounds of resident workgroups.  Every entry of the result is compared with the
f64 oracle, per band of 128 rows (one tile-row) and overall.

References: `oracle.eval_dense` (the plain definition, no property logic) where a dense f64
product is affordable, `oracle.eval_plan` along the same tree (pinned to the dense definition
by the CPU tests) at n = 4096 / 8192, plus `oracle.eval_rows` (the definition again) on one
row of every tile-row."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, I, L, TOL, U, assert_close_by_tiles, rel_fro, structure_mask, upload

pytestmark = pytest.mark.gpu


def one_row_per_tile_row(rows: int, seed: int, tile: int = 128):
    """One row inside every band of `tile` rows, at an offset that varies from band to band."""
    rng = np.random.default_rng(seed)
    picks = [min(r0 + int(rng.integers(0, tile)), rows - 1) for r0 in range(0, rows, tile)]
    return sorted(set(picks) | {0, rows - 1})


def run_whole(dims, props, host, splits=None, flags=0, reference="plan", expect_plan=None, rows_seed=None):
    plan = mom.mom_chain_plan(dims, props) if splits is None else mom.mom_plan_from_splits(dims, props, splits)
    if expect_plan:
        assert plan.string == expect_plan
    if splits is None:
        want_plan = oracle.plan_bruteforce(dims, props)
        assert (plan.cost_mults, plan.splits) == (want_plan["cost"], want_plan["splits"])
    else:
        assert plan.cost_mults == oracle.tree_cost(dims, props, splits)[0]
    dev = upload(host, props, poison=True)
    rows, cols, prop = plan.result
    out = torch.full((rows, cols), float("nan"), device="cuda", dtype=torch.float32)
    ws = torch.full((max(plan.workspace_bytes, 4) // 4,), float("nan"), device="cuda", dtype=torch.float32)
    mom.mom_chain_eval(plan, dev, out=out, workspace=ws, flags=flags)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    np_f = [None if f is None else f.numpy() for f in host]
    if reference == "dense":
        want = oracle.eval_dense(dims, props, np_f)
    else:
        want, want_prop = oracle.eval_plan(dims, props, np_f, plan.splits)
        assert want_prop == prop
    assert_close_by_tiles(got, want, prop)
    mask = structure_mask(prop, rows, cols)
    if prop in (L, U):
        assert np.all(np.isnan(got[~mask])), "other half of a triangular result must stay untouched"
    if rows_seed is not None:          # the property-free definition on one row of every tile-row
        picks = one_row_per_tile_row(rows, rows_seed)
        rows_want = oracle.eval_rows(dims, props, np_f, picks)
        for r, w in zip(picks, rows_want):
            keep = mask[r]
            err = rel_fro(got[r][keep], w[keep])
            assert err <= TOL, "row %d: relative error %.3e" % (r, err)
    return plan


# ---- one dense-checked product per large-launch path ---------------------------------------

@pytest.mark.parametrize("pa,pb", [(L, G), (U, G), (G, L), (G, U)])
def test_single_tiles_second_256_reversed_whole_result(pa, pb):
    # 23 x 23 = 529 tiles of 128, 265 pairs would not fill 256 compute units evenly: single tiles,
    # workgroups 256..511 take tiles 511..256
    n = 2944
    dims, props = [n, n, n], [pa, pb]
    run_whole(dims, props, sc.make_chain(dims, props, 71), reference="dense")


@pytest.mark.parametrize("pa,pb,n", [(L, G, 2900), (U, G, 2899), (G, L, 2899), (G, U, 2900)])
def test_single_tiles_ragged_whole_result(pa, pb, n):
    # 23 x 23 tiles again, the last row and column of tiles ragged (n = 2899: rows not 16-byte aligned
    # either): the tiles of workgroups 256..511 walk their k-range from the far end, so their first
    # chunk is the ragged or the diagonal one
    dims, props = [n, n, n], [pa, pb]
    run_whole(dims, props, sc.make_chain(dims, props, 77), reference="dense")


@pytest.mark.parametrize("dims,props", [([8192, 8192, 4352], [L, G]), ([4352, 8192, 8192], [G, U])])
def test_single_tiles_beyond_four_rounds_whole_result(dims, props):
    # 64 x 34 = 2176 tiles: more than four rounds of resident workgroups
    run_whole(dims, props, sc.make_chain(dims, props, 79))


@pytest.mark.parametrize("pa,pb,n", [(L, G, 4000), (U, G, 3999), (G, L, 3999), (G, U, 4000)])
def test_paired_tiles_ragged_whole_result(pa, pb, n):
    # 32 x 32 = 1024 tiles, 512 pairs (two per compute unit): workgroup b takes tiles b and 1023-b, the
    # second one walked from the far end of its k-range; the last row and column of tiles ragged
    # (n = 3999: rows not 16-byte aligned either)
    dims, props = [n, n, n], [pa, pb]
    run_whole(dims, props, sc.make_chain(dims, props, 80), rows_seed=81)


@pytest.mark.parametrize("pa", [L, U])
def test_single_tiles_rectangular_right_hand_side_whole_result(pa):
    # 24 x 28 = 672 tiles, more tile columns than tile rows
    dims, props = [3072, 3072, 3584], [pa, G]
    run_whole(dims, props, sc.make_chain(dims, props, 75), reference="dense")


@pytest.mark.parametrize("pa,pb,n", [(L, L, 2560), (U, U, 2560), (L, L, 2600), (U, U, 2688)])
def test_two_triangular_operands_on_small_tiles_whole_result(pa, pb, n):
    # 820 to 903 tiles of 64 x 64 (a triangular result of this size runs on the small tiles), single
    # tiles with the second 256 workgroups in reverse; one size ragged
    dims, props = [n, n, n], [pa, pb]
    plan = run_whole(dims, props, sc.make_chain(dims, props, 76), reference="dense")
    assert mom.mom_plan_num_launches(plan) == 1


@pytest.mark.parametrize("dims,props", [([4000, 4000, 200], [U, G]), ([200, 4000, 4000], [G, L]),
                                        ([4000, 4000, 200], [L, G]), ([200, 4000, 4000], [G, U]),
                                        ([3999, 3999, 199], [U, G]), ([199, 3999, 3999], [G, L])])
def test_split_k_with_one_triangular_operand_whole_result(dims, props):
    # fewer than 256 tiles and 125 chunks: split-K; with U * G and G * L every slice of a tile's clipped
    # k-range is walked from its far end, and the last chunk of the range is ragged; the last two cases
    # have nothing 16-byte aligned (4-byte loads)
    plan = run_whole(dims, props, sc.make_chain(dims, props, 78), reference="dense")
    assert mom.mom_plan_num_launches(plan) == 2


@pytest.mark.parametrize("dims", [[3072, 1024, 3072], [3000, 1100, 2900], [3001, 1027, 2999]])
def test_last_round_of_equal_tiles_is_cut_along_k_whole_result(dims):
    # 24 x 24 = 576 (or 24 x 23 = 552) equal tiles of 128: one round of 512 and a few left over; the
    # last tile rows form a sub-product of their own whose tiles are cut into k-slices, in the same
    # launch, and a slice-sum launch follows; ragged and unaligned variants
    props = [G, G]
    plan = run_whole(dims, props, sc.make_chain(dims, props, 82), reference="dense")
    assert mom.mom_plan_num_launches(plan) == 2


def test_persistent_grid_whole_result():
    # 24 x 24 = 576 equal tiles > 512 resident workgroups, k = 288 >= 256: every workgroup
    # strides over the tiles, some take two
    dims, props = [3072, 288, 3072], [G, G]
    run_whole(dims, props, sc.make_chain(dims, props, 72), reference="dense")


def test_persistent_grid_ragged_whole_result():
    dims, props = [3000, 300, 3100], [G, G]
    run_whole(dims, props, sc.make_chain(dims, props, 73), reference="dense")


@pytest.mark.parametrize("pa,pb", [(L, L), (U, U), (L, U), (U, L)])
def test_triangular_pairs_many_rounds_whole_result(pa, pb):
    # 33 x 33 tiles: 561 (tri -> tri, paired) or 1089 (tri.tri -> general, paired) tiles, ragged edge
    n = 4100
    dims, props = [n, n, n], [pa, pb]
    run_whole(dims, props, sc.make_chain(dims, props, 74), reference="plan", rows_seed=5)


# ---- the workloads, every entry ------------------------------------------------------------

def test_trmm4096_whole_result():
    c = sc.CONFIGS["trmm4096"]
    run_whole(c.dims, c.props, sc.make_config("trmm4096"), expect_plan="(0 1)", rows_seed=2)


def test_general5_whole_result_both_trees():
    c = sc.CONFIGS["general5"]
    host = sc.make_config("general5")
    run_whole(c.dims, c.props, host, expect_plan="((0 (1 2)) (3 4))", rows_seed=3)
    run_whole(c.dims, c.props, host, splits=oracle.left_to_right_splits(c.props), expect_plan="((((0 1) 2) 3) 4)")


@pytest.mark.parametrize("splits,text", [(None, "(0 (2 (3 4)))"), ([2, 0, 3], "((0 2) (3 4))"),
                                         ([3, 2, 0], "(((0 2) 3) 4)")])
def test_mixed5_whole_result(splits, text):
    c = sc.CONFIGS["mixed5"]
    run_whole(c.dims, c.props, sc.make_config("mixed5"), splits=splits, expect_plan=text,
              rows_seed=4 if splits is None else None)


def test_lower_times_lower_8192_whole_result():
    # 2080 tiles, unpaired, longest diagonals first: more than four rounds of resident workgroups
    n = 8192
    dims, props = [n, n, n], [L, L]
    plan = run_whole(dims, props, sc.make_chain(dims, props, 40), rows_seed=8)
    assert plan.result == (n, n, L)


def test_lower_times_upper_8192_whole_result():
    # 4096 tiles in shells
    n = 8192
    dims, props = [n, n, n], [L, U]
    run_whole(dims, props, sc.make_chain(dims, props, 44))
