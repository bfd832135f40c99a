"""Helpers of the GPU parity tests: run a chain through the C ABI and compare with the oracle."""
import numpy as np
import torch

import oracle
import paper_2208_10391_amd as mom
import synthetic_chains as sc

G, L, U, I, D = 0, 1, 2, 3, 4
TOL = 1e-4          # max relative Frobenius error against the f64 oracle


def rel_fro(got: np.ndarray, want: np.ndarray) -> float:
    want = want.astype(np.float64)
    denom = np.linalg.norm(want)
    num = np.linalg.norm(got.astype(np.float64) - want)
    return float(num / denom) if denom > 0 else float(num)


def structure_mask(prop: int, rows: int, cols: int) -> np.ndarray:
    ones = np.ones((rows, cols), dtype=bool)
    if prop == L:
        return np.tril(ones)
    if prop == U:
        return np.triu(ones)
    if prop in (I, D):
        return np.eye(rows, cols, dtype=bool)
    return ones


def poison_other_half(t: torch.Tensor, prop: int) -> torch.Tensor:
    """Device copy of a triangular factor whose zero half holds NaN: the library must not let
    it reach a result (it only ever reads the triangle)."""
    if prop not in (L, U, D):
        return t
    nan = torch.full_like(t, float("nan"))
    ones = torch.ones_like(t, dtype=torch.bool)
    keep = torch.tril(ones) if prop == L else torch.triu(ones) if prop == U else torch.tril(torch.triu(ones))
    return torch.where(keep, t, nan)


def upload(factors, props, poison=True, pad_cols=0):
    """Host factors -> device tensors; pad_cols > 0 embeds each in a wider buffer (row stride)."""
    dev = []
    for f, p in zip(factors, props):
        if f is None:
            dev.append(None)
            continue
        d = f.cuda()
        if poison:
            d = poison_other_half(d, p)
        if pad_cols:
            wide = torch.full((d.shape[0], d.shape[1] + pad_cols), float("nan"), device="cuda", dtype=torch.float32)
            wide[:, :d.shape[1]] = d
            d = wide[:, :d.shape[1]]
        dev.append(d)
    return dev


def eval_chain(dims, props, factors, splits=None, flags=0, poison=True, pad_cols=0, out_pad=0, trans=None):
    """Returns (plan, result as numpy with NaN sentinel where nothing was written).  With `trans`
    the factors are the stored matrices (props theirs) and enter the chain transposed where flagged."""
    plan = mom.mom_chain_plan(dims, props, trans=trans) if splits is None else \
        mom.mom_plan_from_splits(dims, props, splits, trans=trans)
    dev = upload(factors, props, poison, pad_cols)
    rows, cols, _ = plan.result
    out_full = torch.full((rows, cols + out_pad), float("nan"), device="cuda", dtype=torch.float32)
    out = out_full[:, :cols]
    mom.mom_chain_eval(plan, dev, out=out, flags=flags)
    torch.cuda.synchronize()
    res = out_full.cpu().numpy()
    if out_pad:
        assert np.all(np.isnan(res[:, cols:])), "wrote beyond the row of the result"
    return plan, res[:, :cols]


def assert_close_by_tiles(got: np.ndarray, want: np.ndarray, prop: int = G, tile: int = 128, tol: float = TOL):
    """Whole-result comparison that localises a bad tile: the relative Frobenius error must hold
    overall AND in every band of `tile` rows (the rows one tile-row of the product kernel
    writes), both restricted to the structure of `prop`; on failure the worst tile x tile block
    is named.  `want` is the f64 reference."""
    rows, cols = want.shape
    mask = structure_mask(prop, rows, cols)
    diff = np.where(mask, got.astype(np.float64) - want, 0.0)
    assert not np.any(np.isnan(diff)), "unwritten entries inside the result's structure"
    ref = np.where(mask, want, 0.0)
    d2, r2 = diff * diff, ref * ref
    scale = np.sqrt(r2.sum() / max(int(mask.sum()), 1))          # rms magnitude of a result entry
    worst = (0.0, -1)
    for r0 in range(0, rows, tile):
        num, den, cnt = d2[r0:r0 + tile].sum(), r2[r0:r0 + tile].sum(), int(mask[r0:r0 + tile].sum())
        # a band of few or tiny entries is measured against the typical entry as well
        err = np.sqrt(num) / max(np.sqrt(den), scale * np.sqrt(cnt) * 1e-3, 1e-300)
        worst = max(worst, (float(err), r0 // tile))
    if worst[0] > tol:
        tr = worst[1]
        band = d2[tr * tile:(tr + 1) * tile]
        per_col = [float(np.sqrt(band[:, c0:c0 + tile].max())) for c0 in range(0, cols, tile)]
        tc = int(np.argmax(per_col))
        raise AssertionError("tile-row %d: relative error %.3e; worst tile (%d, %d), max abs error %.3e" %
                             (tr, worst[0], tr, tc, per_col[tc]))
    total = float(np.sqrt(d2.sum()) / max(np.sqrt(r2.sum()), 1e-300))
    assert total <= tol, "relative Frobenius error %.3e" % total
    return total, worst[0]


def check_against_dense(dims, props, factors, splits=None, flags=0, **kw):
    plan, got = eval_chain(dims, props, factors, splits, flags, **kw)
    np_f = [None if f is None else f.numpy() for f in factors]
    want = oracle.eval_dense(dims, props, np_f, trans=kw.get("trans"))
    rows, cols, prop = plan.result
    mask = structure_mask(prop, rows, cols)
    if prop == I:
        assert np.array_equal(got, np.eye(rows, dtype=np.float32))
        return plan, got
    assert not np.any(np.isnan(got[mask])), "unwritten entries inside the result's structure"
    err = rel_fro(np.where(mask, got, 0.0), np.where(mask, want, 0.0))
    assert err <= TOL, "relative Frobenius error %.3e" % err
    assert_close_by_tiles(got, want, prop)
    if prop in (L, U, D):
        other = got[~mask]
        if flags & mom.MOM_OUT_ZERO_FILL_TRIANGLE:
            assert np.all(other == 0.0), "other half must be zero-filled"
        else:
            assert np.all(np.isnan(other)), "other half of a triangular result must stay untouched"
    return plan, got
