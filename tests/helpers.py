"""Test-side helpers (no GPU, no oracle arithmetic): tree enumeration, golden readers."""
import os
from typing import Iterator, List

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_lines(name: str) -> List[str]:
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.rstrip("\n") for ln in f if ln.strip() and not ln.startswith("#")]


def all_preorder_trees(lo: int, hi: int) -> Iterator[List[int]]:
    """Every binary tree over positions lo..hi as its preorder split list."""
    if lo == hi:
        yield []
        return
    for s in range(lo, hi):
        for left in all_preorder_trees(lo, s):
            for right in all_preorder_trees(s + 1, hi):
                yield [s] + left + right


def random_chain(rng, n: int, max_dim: int, props_pool=(0, 1, 2, 3)):
    """Random dims/props with the squareness that triangular and Identity factors need."""
    props = [int(rng.choice(props_pool)) for _ in range(n)]
    dims = [int(rng.integers(1, max_dim + 1))]
    for p in props:
        dims.append(dims[-1] if p != 0 else int(rng.integers(1, max_dim + 1)))
    return dims, props
