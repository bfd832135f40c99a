"""Seeded synthetic inputs for property-annotated matrix chains.

Shared by the tests, the benchmark, the smoke check and the CPU oracle's callers.
This module holds no arithmetic of the method: it only draws uniform[-1, 1) f32
entries from a seed and writes the zeros a factor's property prescribes, as the
Fill operation of the paper does when it initialises an object (Sec. 2, Table 1).

Properties: 0 general, 1 lowerTri (zeros above the diagonal), 2 upperTri (zeros below
the diagonal), 3 Identity (no buffer at all), 4 diagonal (both triangles' zeros).  The diagonal of a triangular factor is
ordinary data.
"""
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

GENERAL, LOWER_TRI, UPPER_TRI, IDENTITY, DIAGONAL = 0, 1, 2, 3, 4


@dataclass(frozen=True)
class ChainConfig:
    """One workload: factor t is dims[t] x dims[t+1] with property props[t]."""
    name: str
    number: int                 # 1-based workload number, also the seed family
    dims: Sequence[int]
    props: Sequence[int]
    batch: int = 0              # 0 = a single chain; >0 = that many independent chains
    trans: Sequence[int] = ()   # which factors enter transposed (props: of the stored matrices); () = none


CONFIGS = {
    # tiny chain: lowerTri 64x64, general 64x32, general 32x128
    "tiny": ChainConfig("tiny", 1, (64, 64, 32, 128), (LOWER_TRI, GENERAL, GENERAL)),
    # one triangular-times-general product, n = 4096
    "trmm4096": ChainConfig("trmm4096", 2, (4096, 4096, 4096), (LOWER_TRI, GENERAL)),
    # the same product with both buffers holding transposes: (stored upperTri)^T * (stored G)^T
    "trmm4096_transposed": ChainConfig("trmm4096_transposed", 2, (4096, 4096, 4096), (UPPER_TRI, GENERAL), trans=(1, 1)),
    # order-sensitive chain of five general factors
    "general5": ChainConfig("general5", 3, (8192, 512, 8192, 64, 4096, 2048), (GENERAL,) * 5),
    # L1 * I * L2 * U * G
    "mixed5": ChainConfig("mixed5", 4, (8192, 8192, 8192, 8192, 8192, 1024),
                          (LOWER_TRI, IDENTITY, LOWER_TRI, UPPER_TRI, GENERAL)),
    # general * general * general * lowerTri: a chain on which the multiplication count and the
    # time model choose different trees (the count forms the 1024 x 256 product with k = 4096
    # first, then two more dependent products; the time model pairs the factors up, two
    # independent products that share a launch, at 1.29 times the multiplications)
    "gggl256": ChainConfig("gggl256", 6, (256, 1024, 4096, 256, 256), (GENERAL, GENERAL, GENERAL, LOWER_TRI)),
    # 4096 independent chains L * G * U of 32x32 factors
    "batched32": ChainConfig("batched32", 5, (32, 32, 32, 32), (LOWER_TRI, GENERAL, UPPER_TRI),
                             batch=4096),
}


def factor_seed(config_number: int, factor_index: int) -> int:
    return 1000 * config_number + factor_index


def make_factor(rows: int, cols: int, prop: int, seed: int, batch: int = 0) -> Optional[torch.Tensor]:
    """Uniform[-1, 1) f32 matrix (or [batch, rows, cols] stack) on the CPU with the zeros of
    `prop` written; None for an Identity factor, which has no buffer."""
    if prop == IDENTITY:
        return None
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    shape = (batch, rows, cols) if batch > 0 else (rows, cols)
    a = torch.rand(shape, generator=g, dtype=torch.float32) * 2.0 - 1.0
    if prop == LOWER_TRI:
        a = torch.tril(a)
    elif prop == UPPER_TRI:
        a = torch.triu(a)
    elif prop == DIAGONAL:
        a = torch.tril(torch.triu(a))
    elif prop != GENERAL:
        raise ValueError("unknown property %r" % (prop,))
    return a.contiguous()


def make_chain(dims: Sequence[int], props: Sequence[int], seed_family: int,
               batch: int = 0, trans: Optional[Sequence[int]] = None) -> List[Optional[torch.Tensor]]:
    """All factors of one chain; factor t is drawn from seed 1000*seed_family + t.  Where
    trans[t] is set the chain holds the transpose of what is stored (Table 1, Transpose): the
    buffer drawn is the dims[t+1] x dims[t] matrix, and props[t] is the property of that
    stored matrix."""
    assert len(dims) == len(props) + 1
    out = []
    for t in range(len(props)):
        r, c = (dims[t + 1], dims[t]) if (trans is not None and trans[t]) else (dims[t], dims[t + 1])
        out.append(make_factor(r, c, props[t], factor_seed(seed_family, t), batch))
    return out


def make_config(name: str) -> List[Optional[torch.Tensor]]:
    c = CONFIGS[name]
    return make_chain(c.dims, c.props, c.number, c.batch, list(c.trans) if c.trans else None)
