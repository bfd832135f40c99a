"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc
from gpu_util import G, I, L, TOL, U, check_against_dense, eval_chain, rel_fro, structure_mask, upload
from helpers import all_preorder_trees, golden_lines, random_chain

pytestmark = pytest.mark.gpu


def chain(dims, props, family):
    return sc.make_chain(dims, props, family)


def test_paper_listing_5x5_lower_times_lower():
    lines = golden_lines("listing_5x5_lower_lower.txt")
    want = np.array([[float(x) for x in ln.split()] for ln in lines[2:]], dtype=np.float32)
    a = torch.tril(torch.ones(5, 5))
    plan, got = eval_chain([5, 5, 5], [L, L], [a, a.clone()])
    assert plan.result == (5, 5, L)
    low = np.tril(np.ones((5, 5), dtype=bool))
    assert np.array_equal(got[low], want[low])            # small integers: exact in f32
    assert np.all(np.isnan(got[~low]))                    # only the triangle is written
    _, full = eval_chain([5, 5, 5], [L, L], [a, a.clone()], flags=mom.MOM_OUT_ZERO_FILL_TRIANGLE)
    assert np.array_equal(full, want)


def test_workload_tiny():
    c = sc.CONFIGS["tiny"]
    plan, _ = check_against_dense(c.dims, c.props, sc.make_config("tiny"))
    assert plan.string == "((0 1) 2)"


@pytest.mark.parametrize("pa", [G, L, U])
@pytest.mark.parametrize("pb", [G, L, U])
@pytest.mark.parametrize("n", [1, 33, 130, 257, 300])
def test_every_property_pair(pa, pb, n):
    # several 128- and 64-wide tiles plus a ragged tail; unaligned rows for odd n
    m = n if pa != G else n + 7
    c = n if pb != G else max(n - 5, 1)
    dims, props = [m, n, c], [pa, pb]
    check_against_dense(dims, props, chain(dims, props, 300 + n))


@pytest.mark.parametrize("pa", [G, L, U])
@pytest.mark.parametrize("pb", [G, L, U])
@pytest.mark.parametrize("n", [128, 256, 384, 640])
def test_every_property_pair_whole_tiles(pa, pb, n):
    # nothing ragged: every tile takes 16-byte loads, the long k-ranges run the steady-state
    # chunk body in pairs, diagonals are masked when staged, and k-ranges of 4, 8, 12, ...
    # chunks start the pairs at either parity
    dims, props = [n, n, n], [pa, pb]
    check_against_dense(dims, props, chain(dims, props, 900 + n))


@pytest.mark.parametrize("k", [32, 64, 96, 160, 224, 288])
def test_short_k_ranges_of_whole_tiles(k):
    # 1, 2, 3, 5, 7, 9 chunks per tile, several tiles per workgroup never: one launch, 2x3 tiles
    dims, props = [256, k, 384], [G, G]
    check_against_dense(dims, props, chain(dims, props, 950 + k))


def test_split_k_with_empty_slices():
    # 400 chunks of 32 over 48 slices of 9: the last slices get no chunk and write zeros
    dims, props = [512, 12800, 64], [G, G]
    check_against_dense(dims, props, chain(dims, props, 960))


@pytest.mark.parametrize("pa,pb", [(L, L), (U, U), (L, U), (U, L), (L, G), (G, U)])
def test_zero_fill_flag_and_strided_buffers(pa, pb):
    n = 200
    dims, props = [n, n, n], [pa, pb]
    check_against_dense(dims, props, chain(dims, props, 41), flags=mom.MOM_OUT_ZERO_FILL_TRIANGLE,
                        pad_cols=12, out_pad=20)
    check_against_dense(dims, props, chain(dims, props, 42), pad_cols=3, out_pad=1)


@pytest.mark.parametrize("m,k,n", [(33, 65, 17), (128, 128, 128), (129, 16, 127), (64, 1000, 64),
                                   (500, 40, 700), (1, 1, 1), (256, 17, 384), (70, 300, 1)])
def test_general_product_shapes(m, k, n):
    dims, props = [m, k, n], [G, G]
    check_against_dense(dims, props, chain(dims, props, 500 + m))


@pytest.mark.parametrize("m,k,n", [(64, 5000, 64), (130, 2000, 70), (33, 4097, 17), (512, 8192, 64), (64, 4096, 2048)])
def test_long_k_products_are_split(m, k, n):
    # few output tiles and a long k: the k-range is cut into slices that a second kernel sums
    dims, props = [m, k, n], [G, G]
    check_against_dense(dims, props, chain(dims, props, 700 + m))


def test_independent_products_share_a_launch():
    # ((A B) (C D)) and (((A B) (C D)) ((E F) (G H))): products of one level run side by side,
    # each with its own temporaries and split-K scratch
    dims, props = [96, 1500, 80, 1200, 72], [G, G, G, G]
    f = chain(dims, props, 810)
    plan, _ = check_against_dense(dims, props, f, splits=[1, 0, 2])
    assert plan.string == "((0 1) (2 3))"
    dims, props = [70, 900, 64, 64, 64, 1000, 90, 700, 33], [G, G, L, U, G, G, G, G]
    f = chain(dims, props, 820)
    plan, _ = check_against_dense(dims, props, f, splits=[3, 1, 0, 2, 5, 4, 6])
    assert plan.string == "(((0 1) (2 3)) ((4 5) (6 7)))"


def test_paper_sec4_chain_both_trees():
    kv = dict(ln.split(" ", 1) for ln in golden_lines("sec4_chain.txt"))
    dims = [int(x) for x in kv["dims"].split()]
    props = [G] * 4
    f = chain(dims, props, 174)
    plan, a = check_against_dense(dims, props, f)
    assert plan.string == kv["chosen"]
    plan2, b = check_against_dense(dims, props, f, splits=oracle.left_to_right_splits(props))
    assert plan2.string == kv["initial"]
    assert rel_fro(a, b) <= 2 * TOL


def test_identity_rules_bit_exact():
    a = sc.make_factor(70, 70, G, 9)
    for dims, props, fac in (([70] * 3, [G, I], [a, None]), ([70] * 3, [I, G], [None, a]),
                             ([70] * 4, [I, G, I], [None, a, None])):
        plan, got = eval_chain(dims, props, fac)
        assert mom.mom_plan_num_products(plan) == 0
        assert np.array_equal(got, a.numpy())              # A * I = A is a copy
    lo = sc.make_factor(70, 70, L, 10)
    plan, got = eval_chain([70] * 3, [L, I], [lo, None])
    low = np.tril(np.ones((70, 70), dtype=bool))
    assert plan.result == (70, 70, L)
    assert np.array_equal(got[low], lo.numpy()[low]) and np.all(np.isnan(got[~low]))
    plan, got = eval_chain([9] * 3, [I, I], [None, None])
    assert plan.result == (9, 9, I) and np.array_equal(got, np.eye(9, dtype=np.float32))


def test_every_tree_of_a_mixed_chain():
    dims, props = [90, 90, 90, 90, 90, 50], [L, I, L, U, G]
    f = chain(dims, props, 77)
    surv = oracle.survivors(props)
    results = []
    for tree in all_preorder_trees(0, len(surv) - 1):
        splits = [surv[s] for s in tree]
        plan, got = check_against_dense(dims, props, f, splits=splits)
        assert plan.cost_mults == oracle.tree_cost(dims, props, splits)[0]
        results.append(got)
    assert len(results) == 5


def test_random_chains_with_random_properties():
    rng = np.random.default_rng(99)
    for trial in range(40):
        n = int(rng.integers(1, 7))
        dims, props = random_chain(rng, n, 180)
        f = chain(dims, props, 600 + trial)
        plan, _ = check_against_dense(dims, props, f, flags=int(rng.integers(0, 2)))
        want = oracle.plan_bruteforce(dims, props)
        assert (plan.cost_mults, plan.splits) == (want["cost"], want["splits"])


def test_random_chains_larger_and_snapped_to_tiles():
    """Larger random chains, half of them snapped to multiples of 32 / 64 / 128 (16-byte paths),
    random forced trees, strided buffers."""
    rng = np.random.default_rng(123)
    for trial in range(40):
        n = int(rng.integers(1, 5))
        dims, props = random_chain(rng, n, int(rng.choice([96, 300, 700])))
        if rng.integers(0, 2):
            snap = int(rng.choice([32, 64, 128]))
            dims = [max(snap, (d // snap) * snap) for d in dims]
            for t, p in enumerate(props):
                if p != G:
                    dims[t + 1] = dims[t]
        f = chain(dims, props, 5000 + trial)
        surv = oracle.survivors(props)
        splits = None
        if len(surv) >= 3 and rng.integers(0, 2):
            trees = list(all_preorder_trees(0, len(surv) - 1))
            splits = [surv[x] for x in trees[int(rng.integers(0, len(trees)))]]
        pad = int(rng.choice([0, 0, 4, 5]))
        check_against_dense(dims, props, f, splits=splits, flags=int(rng.integers(0, 2)), pad_cols=pad, out_pad=pad)


def test_triangular_temporaries_feed_masked_products():
    # (L1 L2) is a lowerTri temporary of which only the triangle is written; whatever the
    # workspace held before must not leak into ((L1 L2) U) G
    n = 260
    dims, props = [n, n, n, n, 40], [L, L, U, G]
    f = chain(dims, props, 88)
    plan = mom.mom_plan_from_splits(dims, props, [2, 1, 0])
    assert plan.string == "(((0 1) 2) 3)"
    dev = upload(f, props)
    ws = torch.full((plan.workspace_bytes // 4,), float("nan"), device="cuda", dtype=torch.float32)
    out = mom.mom_chain_eval(plan, dev, workspace=ws)
    torch.cuda.synchronize()
    want = oracle.eval_dense(dims, props, [x.numpy() for x in f])
    assert rel_fro(out.cpu().numpy(), want) <= TOL


def test_eval_argument_errors_on_device():
    p = mom.mom_chain_plan([64, 64, 64, 64], [G, G, G])
    f = [torch.zeros(64, 64, device="cuda") for _ in range(3)]
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(mom.MomError):
        mom.mom_chain_eval(p, f, workspace=small)
    with pytest.raises(ValueError):
        mom.mom_chain_eval(p, f[:2])
    with pytest.raises(TypeError):
        mom.mom_chain_eval(p, [x.cpu() for x in f])


def test_bound_call_can_be_enqueued_again():
    """Arguments marshalled once: every later call of the bound object is the same evaluation."""
    dims, props = [130, 70, 70, 45], [G, L, G]
    host = chain(dims, props, 77)
    want = oracle.eval_dense(dims, props, [f.numpy() for f in host])
    plan = mom.mom_chain_plan(dims, props)
    call = mom.bind_chain_eval(plan, upload(host, props))
    for _ in range(3):
        call.out.fill_(float("nan"))
        got = call().cpu().numpy()
        assert rel_fro(got, want) <= TOL

    bdims, bprops, batch = [32, 32, 32, 32], [L, G, U], 9
    bhost = [sc.make_factor(32, 32, p, 500 + t, batch) for t, p in enumerate(bprops)]
    bplan = mom.mom_chain_plan(bdims, bprops)
    bcall = mom.bind_chain_eval_batched(bplan, [f.cuda() for f in bhost])
    for _ in range(3):
        bcall.out.fill_(float("nan"))
        got = bcall().cpu().numpy()
        for b in range(batch):
            w = oracle.eval_dense(bdims, bprops, [f[b].numpy() for f in bhost])
            assert rel_fro(got[b], w) <= TOL


def test_mfma_probe_runs_and_counts_its_flop():
    sink = torch.zeros(256, device="cuda")
    flop = mom.mom_probe_mfma_peak(10, sink)
    torch.cuda.synchronize()
    assert flop == 512 * 4 * 10 * 32 * 4096.0       # workgroups x wavefronts x trips x MFMAs x 2*32*32*2
    assert float(sink.abs().sum()) == 0.0           # the sink is never written
    with pytest.raises(mom.MomError):
        mom.mom_probe_mfma_peak(0, sink)


def test_evaluation_can_be_captured_in_a_graph_and_replayed():
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so an
    evaluation records into a HIP graph; every replay, with eager work in between, must
    reproduce the eager result bit for bit (same kernels, same order of summation)."""
    dims, props = [96, 1500, 80, 1200, 72], [G, G, G, G]          # fused level + split-K + slice sum
    host = chain(dims, props, 830)
    plan = mom.mom_plan_from_splits(dims, props, [1, 0, 2])
    dev = upload(host, props)
    call = mom.bind_chain_eval(plan, dev)
    eager = call().clone()                                         # also the warm-up before capture
    torch.cuda.synchronize()
    want = oracle.eval_dense(dims, props, [f.numpy() for f in host])
    assert rel_fro(eager.cpu().numpy(), want) <= TOL
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        call()
        torch.cuda.synchronize()
        with torch.cuda.graph(graph, stream=side):
            call()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(4):
        call.out.fill_(float("nan"))
        other = (dev[0] @ dev[0].t()).sum()                        # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(call.out, eager), "replay %d differs" % rep
        assert torch.isfinite(other)


FIRST_USE_UNDER_CAPTURE = r"""
import sys
import torch
sys.path.insert(0, %r)
import paper_2208_10391_amd as mom
from paper_2208_10391_amd import binding
a = torch.rand(200, 200, device="cuda")
b = torch.rand(200, 200, device="cuda")
plan = mom.mom_chain_plan([200, 200, 200], [0, 0])
call = mom.bind_chain_eval(plan, [a, b])
side = torch.cuda.Stream()
side.wait_stream(torch.cuda.current_stream())
torch.cuda.synchronize()
graph = torch.cuda.CUDAGraph()
status = None
with torch.cuda.stream(side):
    with torch.cuda.graph(graph, stream=side):
        try:
            call()                      # the very first evaluation of this process: refused
        except mom.MomError as e:
            status = binding.STATUS_NAMES[e.status]
assert status == "MOM_ERR_NOT_READY", status
mom.mom_init()
graph2 = torch.cuda.CUDAGraph()
with torch.cuda.stream(side):
    with torch.cuda.graph(graph2, stream=side):
        call()                          # after mom_init the first evaluation may be captured
torch.cuda.current_stream().wait_stream(side)
call.out.fill_(float("nan"))
torch.cuda.synchronize()
graph2.replay()
torch.cuda.synchronize()
ref = (a.double() @ b.double())
err = float(torch.linalg.norm(call.out.double() - ref) / torch.linalg.norm(ref))
assert err <= 1e-4, err
print("capture ok", status, err)
"""


def test_first_evaluation_under_capture_returns_a_status_and_mom_init_makes_it_legal():
    """In a fresh process (the per-device set-up has not happened yet) a first evaluation on a
    capturing stream must come back as MOM_ERR_NOT_READY with the capture intact; after
    mom_init the same call records and replays."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, "-c", FIRST_USE_UNDER_CAPTURE % root], capture_output=True, text=True, timeout=240)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "capture ok MOM_ERR_NOT_READY" in r.stdout


@pytest.mark.parametrize("pa,pb", [(L, G), (U, G), (G, L), (G, U), (L, U), (U, L)])
def test_few_tiles_with_triangular_operands_are_split_along_k(pa, pb):
    # a general result on few tiles and a long k: every tile's own (clipped) k-range is dealt out
    # to slices, the short tiles near the tip of the triangle leave some slices empty
    n = 2304
    dims = [n, n, 100] if pb == G else ([70, n, n] if pa == G else [n, n, n])
    if pa != G and pb != G:
        n = 1100                                   # 9 x 9 = 81 tiles of L*U / U*L
        dims = [n, n, n]
    props = [pa, pb]
    plan, _ = check_against_dense(dims, props, chain(dims, props, 970))
    # 72 chunks in the full k for n = 2304: product launch + slice sum; 35 chunks for n = 1100: one launch
    assert mom.mom_plan_num_launches(plan) == (2 if n == 2304 else 1)


def test_row_stride_beyond_the_reach_of_32_bit_offsets():
    """A factor whose rows lie 2^22 elements (16 MiB) apart: the 16-byte loads of the product kernel
    address a chunk with 32-bit byte offsets from its first element, which 128 such rows exceed, so
    these operands take the element-wise path with 64-bit addresses."""
    m, k, n, ld = 200, 160, 136, 1 << 22
    a = sc.make_factor(m, k, G, 31)
    b = sc.make_factor(k, n, G, 32)
    wide = torch.empty((m - 1) * ld + k, device="cuda", dtype=torch.float32)          # 3.3 GB, only m x k of it used
    a_dev = torch.as_strided(wide, (m, k), (ld, 1))
    a_dev.copy_(a.cuda())
    plan = mom.mom_chain_plan([m, k, n], [G, G])
    out = mom.mom_chain_eval(plan, [a_dev, b.cuda()])
    torch.cuda.synchronize()
    want = a.numpy().astype(np.float64) @ b.numpy().astype(np.float64)
    assert rel_fro(out.cpu().numpy(), want) <= TOL
    # and as the right-hand operand, transposed
    plan = mom.mom_chain_plan_ex([n, k, m], [G, G], [1, 1])
    out = mom.mom_chain_eval(plan, [b.cuda(), a_dev])
    torch.cuda.synchronize()
    assert rel_fro(out.cpu().numpy(), want.T) <= TOL
    del wide, a_dev
    torch.cuda.empty_cache()


@pytest.mark.parametrize("dims", [[128, 130, 62], [128, 130, 192], [256, 258, 254], [2944, 130, 2814]])
def test_aligned_row_stride_with_extents_that_are_not_multiples_of_four(dims):
    # two NaN-filled columns of padding make every row stride a multiple of four while the extents are
    # not: interior tiles load 16 bytes at a time and the group that straddles the end of k is cut by
    # the descriptor in the matrix's last row (its tail lies past the last element) and by the staging
    # mask elsewhere; tiles that poke over the right edge load 4 bytes at a time.  The last case takes
    # the 128 x 128 tiles.
    check_against_dense(dims, [G, G], sc.make_chain(dims, [G, G], 4100 + dims[0]), pad_cols=2)
