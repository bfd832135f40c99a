"""CPU f64 oracle for property-annotated matrix-chain products.

TEST INFRASTRUCTURE ONLY: the tests, the smoke check and the benchmark's CPU
baseline are the only callers.  Nothing here is shared with, or imported by,
the GPU library, and the GPU library never falls back to it.

Thin ctypes layer over oracle.c; every function documents the passage of the
paper (MOM: Matrix Operations in MLIR) that it states.  Properties are the
integers 0 general, 1 lowerTri, 2 upperTri, 3 Identity, 4 diagonal = {lowerTri, upperTri} (Sec. 2).
"""
import ctypes
from typing import List, Optional, Sequence, Tuple

import numpy as np

from .build import build as _build

GENERAL, LOWER_TRI, UPPER_TRI, IDENTITY, DIAGONAL = 0, 1, 2, 3, 4

_lib = ctypes.CDLL(_build())

_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_f64p = ctypes.POINTER(ctypes.c_double)
_fpp = ctypes.POINTER(ctypes.c_void_p)

_lib.oracle_count_mults.restype = ctypes.c_uint64
_lib.oracle_count_mults.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                    ctypes.c_int32, ctypes.c_int32]
_lib.oracle_plan_bruteforce.restype = ctypes.c_int
_lib.oracle_plan_bruteforce.argtypes = [ctypes.c_int32, _i64p, _i32p, ctypes.c_int32,
                                        ctypes.POINTER(ctypes.c_uint64), _i32p, _i32p, _i32p,
                                        ctypes.POINTER(ctypes.c_int64)]
_lib.oracle_tree_cost.restype = ctypes.c_int
_lib.oracle_tree_cost.argtypes = [ctypes.c_int32, _i64p, _i32p, _i32p,
                                  ctypes.POINTER(ctypes.c_uint64), _i32p]
_lib.oracle_eval_dense_t.restype = ctypes.c_int
_lib.oracle_eval_dense_t.argtypes = [ctypes.c_int32, _i64p, _i32p, _i32p, _fpp, _f64p]
_lib.oracle_eval_rows_t.restype = ctypes.c_int
_lib.oracle_eval_rows_t.argtypes = [ctypes.c_int32, _i64p, _i32p, _i32p, _fpp, ctypes.c_int32, _i64p, _f64p]
_lib.oracle_eval_plan_t.restype = ctypes.c_int
_lib.oracle_eval_plan_t.argtypes = [ctypes.c_int32, _i64p, _i32p, _i32p, _fpp, _i32p, _f64p, _i32p]
_lib.oracle_transposed_property.restype = ctypes.c_int32
_lib.oracle_transposed_property.argtypes = [ctypes.c_int32]
_lib.oracle_product_time_ps.restype = ctypes.c_uint64
_lib.oracle_product_time_ps.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, ctypes.c_int32]
_lib.oracle_plan_bruteforce_time.restype = ctypes.c_int
_lib.oracle_plan_bruteforce_time.argtypes = [ctypes.c_int32, _i64p, _i32p, ctypes.POINTER(ctypes.c_uint64),
                                             ctypes.POINTER(ctypes.c_uint64), _i32p, _i32p]
_lib.oracle_tree_time.restype = ctypes.c_int
_lib.oracle_tree_time.argtypes = [ctypes.c_int32, _i64p, _i32p, _i32p, ctypes.POINTER(ctypes.c_uint64)]
_lib.oracle_sum_property.restype = ctypes.c_int32
_lib.oracle_sum_property.argtypes = [ctypes.c_int32, _i32p]
_lib.oracle_add_dense.restype = ctypes.c_int
_lib.oracle_add_dense.argtypes = [ctypes.c_int64, ctypes.c_int64, ctypes.c_int32, _i32p, _i32p, _fpp, _f64p]
_lib.oracle_max_threads.restype = ctypes.c_int


def _dims(dims) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(dims, dtype=np.int64))


def _props(props) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(props, dtype=np.int32))


def _trans(trans, n: int):
    """None -> NULL pointer (no factor transposed), else n flags."""
    if trans is None:
        return None, None
    t = np.ascontiguousarray(np.asarray([1 if x else 0 for x in trans], dtype=np.int32))
    assert len(t) == n
    return t.ctypes.data_as(_i32p), t


def transposed_property(prop: int) -> int:
    """Property of the transpose: lowerTri(A) -> upperTri(A^T) and back (the inference rule of
    Sec. 2, Transformations); general and Identity are unchanged."""
    return int(_lib.oracle_transposed_property(int(prop)))


def chain_props(props, trans=None) -> List[int]:
    """Properties the factors have inside the chain: a transposed factor's stored property mirrored."""
    if trans is None:
        return [int(p) for p in props]
    return [transposed_property(p) if t else int(p) for p, t in zip(props, trans)]


def _factor_ptrs(dims: np.ndarray, props: np.ndarray, factors: Sequence[Optional[np.ndarray]], trans=None):
    """Host f32 row-major buffers -> array of pointers (Identity entries may be None).  The buffer
    of a transposed factor holds the dims[t+1] x dims[t] matrix whose transpose enters the chain."""
    keep = []
    ptrs = (ctypes.c_void_p * len(props))()
    for t, p in enumerate(props):
        f = factors[t]
        if f is None:
            if p != IDENTITY:
                raise ValueError("factor %d has no buffer but is not an Identity" % t)
            ptrs[t] = None
            continue
        a = np.ascontiguousarray(np.asarray(f, dtype=np.float32))
        want = (dims[t + 1], dims[t]) if (trans is not None and trans[t]) else (dims[t], dims[t + 1])
        if a.shape != want:
            raise ValueError("factor %d has shape %s, expected %s" % (t, a.shape, want))
        keep.append(a)
        ptrs[t] = a.ctypes.data
    return ptrs, keep


def max_threads() -> int:
    return int(_lib.oracle_max_threads())


def count_mults(m: int, k: int, n: int, pX: int, pY: int) -> int:
    """Scalar products of X(m x k)*Y(k x n) with no structurally-zero operand, counted one
    by one in a triple loop (the planner's cost unit, Sec. 2 Transformations)."""
    return int(_lib.oracle_count_mults(m, k, n, pX, pY))


def plan_bruteforce(dims, props, elide: bool = True, trans=None) -> dict:
    """Minimum-multiplication parenthesisation by enumerating every binary tree
    (Sec. 2: variadic Mul -> binary products with an optimal parenthesisation; matrix-chain
    reordering generalised to properties; identity simplification).

    Returns cost, n_eff, splits (preorder, original factor indices), result_prop, num_trees.
    Ties go to the lexicographically smallest preorder split list.  With `trans`, props are the
    stored properties and the search runs on the properties the factors have inside the chain
    (Table 1 Transpose; Sec. 2 Transformations: lowerTri(A) -> upperTri(A^T))."""
    d, p = _dims(dims), _props(chain_props(props, trans))
    n = len(p)
    assert len(d) == n + 1
    cost = ctypes.c_uint64()
    neff = ctypes.c_int32()
    rprop = ctypes.c_int32()
    ntrees = ctypes.c_int64()
    splits = np.zeros(max(n, 1), dtype=np.int32)
    rc = _lib.oracle_plan_bruteforce(n, d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p), int(elide),
                                     ctypes.byref(cost), ctypes.byref(neff),
                                     splits.ctypes.data_as(_i32p), ctypes.byref(rprop),
                                     ctypes.byref(ntrees))
    if rc != 0:
        raise OverflowError("cost does not fit in 64 bits")
    k = max(neff.value - 1, 0)
    return {"cost": int(cost.value), "n_eff": int(neff.value), "splits": [int(x) for x in splits[:k]],
            "result_prop": int(rprop.value), "num_trees": int(ntrees.value)}


def product_time_ps(m: int, k: int, n: int, pX: int, pY: int) -> int:
    """Modelled time, in picoseconds, of one tiled product on the GPU (the opt-in objective that
    Sec. 4's gap between multiplication count and run time motivates; stated in oracle.c)."""
    return int(_lib.oracle_product_time_ps(m, k, n, pX, pY))


def plan_bruteforce_time(dims, props, trans=None) -> dict:
    """The tree with the smallest modelled time, by enumerating every tree.  Returns time_ps,
    mults (of that tree), n_eff, splits."""
    d, p = _dims(dims), _props(chain_props(props, trans))
    n = len(p)
    t, mu, neff = ctypes.c_uint64(), ctypes.c_uint64(), ctypes.c_int32()
    splits = np.zeros(max(n, 1), dtype=np.int32)
    rc = _lib.oracle_plan_bruteforce_time(n, d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p), ctypes.byref(t),
                                          ctypes.byref(mu), ctypes.byref(neff), splits.ctypes.data_as(_i32p))
    if rc != 0:
        raise OverflowError("a sum does not fit in 64 bits")
    k = max(neff.value - 1, 0)
    return {"time_ps": int(t.value), "mults": int(mu.value), "n_eff": int(neff.value),
            "splits": [int(x) for x in splits[:k]]}


def tree_time_ps(dims, props, splits, trans=None) -> int:
    """Modelled time of one given tree: the sum over its products."""
    d, p = _dims(dims), _props(chain_props(props, trans))
    s = np.ascontiguousarray(np.asarray(list(splits) + [0], dtype=np.int32))
    t = ctypes.c_uint64()
    rc = _lib.oracle_tree_time(len(p), d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p),
                               s.ctypes.data_as(_i32p), ctypes.byref(t))
    if rc == 1:
        raise OverflowError("time does not fit in 64 bits")
    if rc == 2:
        raise ValueError("malformed split list")
    return int(t.value)


def tree_cost(dims, props, splits, trans=None) -> Tuple[int, int]:
    """(cost in scalar multiplications, result property) of one given tree."""
    d, p = _dims(dims), _props(chain_props(props, trans))
    s = np.ascontiguousarray(np.asarray(list(splits) + [0], dtype=np.int32))
    cost = ctypes.c_uint64()
    rprop = ctypes.c_int32()
    rc = _lib.oracle_tree_cost(len(p), d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p),
                               s.ctypes.data_as(_i32p), ctypes.byref(cost), ctypes.byref(rprop))
    if rc == 1:
        raise OverflowError("cost does not fit in 64 bits")
    if rc == 2:
        raise ValueError("malformed split list")
    return int(cost.value), int(rprop.value)


def survivors(props) -> List[int]:
    """Original indices of the factors left after identity simplification (A*I -> A)."""
    return [i for i, p in enumerate(props) if p != IDENTITY]


def plan_string(props, splits) -> str:
    """Parenthesised form of a preorder split list, original indices, e.g. '(0 (2 (3 4)))'."""
    surv = survivors(props)
    if not surv:
        return "I"
    it = iter(splits)

    def rec(lo: int, hi: int) -> str:
        if lo == hi:
            return str(surv[lo])
        s = surv.index(next(it))
        return "(" + rec(lo, s) + " " + rec(s + 1, hi) + ")"

    return rec(0, len(surv) - 1)


def left_to_right_splits(props) -> List[int]:
    """Preorder splits of (((A0 A1) A2) ...), the paper's 'initial parenthesization' (Sec. 4)."""
    surv = survivors(props)
    return [surv[i] for i in range(len(surv) - 2, -1, -1)]


def eval_dense(dims, props, factors, trans=None) -> np.ndarray:
    """The chain product by its plain definition: dense f64 triple loops, left to right,
    Identity materialised as eye, no property logic (Sec. 2, bufferization and Types).
    trans[t] true: factors[t] is the dims[t+1] x dims[t] buffer whose transpose is factor t
    (Table 1, Transpose)."""
    d, p = _dims(dims), _props(props)
    ptrs, keep = _factor_ptrs(d, p, factors, trans)
    tp, tkeep = _trans(trans, len(p))
    out = np.zeros((d[0], d[-1]), dtype=np.float64)
    rc = _lib.oracle_eval_dense_t(len(p), d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p), tp,
                                  ctypes.cast(ptrs, _fpp), out.ctypes.data_as(_f64p))
    if rc != 0:
        raise ValueError("oracle_eval_dense failed: %d" % rc)
    del keep
    return out


def eval_rows(dims, props, factors, rows, trans=None) -> np.ndarray:
    """Selected rows of the dense chain product: A_0[r,:] pushed through the other factors."""
    d, p = _dims(dims), _props(props)
    ptrs, keep = _factor_ptrs(d, p, factors, trans)
    tp, tkeep = _trans(trans, len(p))
    r = np.ascontiguousarray(np.asarray(rows, dtype=np.int64))
    out = np.zeros((len(r), d[-1]), dtype=np.float64)
    rc = _lib.oracle_eval_rows_t(len(p), d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p), tp,
                                 ctypes.cast(ptrs, _fpp), len(r), r.ctypes.data_as(_i64p),
                                 out.ctypes.data_as(_f64p))
    if rc != 0:
        raise ValueError("oracle_eval_rows failed: %d" % rc)
    del keep
    return out


def eval_plan(dims, props, factors, splits, trans=None) -> Tuple[np.ndarray, int]:
    """Evaluate along a given tree with loops restricted by the operand properties, f64.
    Returns (dense result, result property).  With `trans`, props describe the stored matrices."""
    d, p = _dims(dims), _props(props)
    ptrs, keep = _factor_ptrs(d, p, factors, trans)
    tp, tkeep = _trans(trans, len(p))
    s = np.ascontiguousarray(np.asarray(list(splits) + [0], dtype=np.int32))
    out = np.zeros((d[0], d[-1]), dtype=np.float64)
    rprop = ctypes.c_int32()
    rc = _lib.oracle_eval_plan_t(len(p), d.ctypes.data_as(_i64p), p.ctypes.data_as(_i32p), tp,
                                 ctypes.cast(ptrs, _fpp), s.ctypes.data_as(_i32p),
                                 out.ctypes.data_as(_f64p), ctypes.byref(rprop))
    if rc != 0:
        raise ValueError("malformed split list")
    del keep
    return out, int(rprop.value)


def sum_property(props, trans=None) -> int:
    """Property of a sum of terms (Table 1, Add): the smallest structure that holds every term's."""
    p = _props(chain_props(props, trans))
    return int(_lib.oracle_sum_property(len(p), p.ctypes.data_as(_i32p)))


def add_dense(rows: int, cols: int, props, terms, trans=None) -> np.ndarray:
    """The variadic Add by its plain definition: entry-wise f64 sum of the terms in their order
    (Table 1, Add; Sec. 2, Operations).  A transposed term is stored cols x rows; Identity is eye."""
    p = _props(props)
    n = len(p)
    keep = []
    ptrs = (ctypes.c_void_p * n)()
    for t in range(n):
        if terms[t] is None:
            if p[t] != IDENTITY:
                raise ValueError("term %d has no buffer but is not an Identity" % t)
            ptrs[t] = None
            continue
        a = np.ascontiguousarray(np.asarray(terms[t], dtype=np.float32))
        want = (cols, rows) if (trans is not None and trans[t]) else (rows, cols)
        if a.shape != want:
            raise ValueError("term %d has shape %s, expected %s" % (t, a.shape, want))
        keep.append(a)
        ptrs[t] = a.ctypes.data
    tp, tkeep = _trans(trans, n)
    out = np.zeros((rows, cols), dtype=np.float64)
    rc = _lib.oracle_add_dense(rows, cols, n, p.ctypes.data_as(_i32p), tp, ctypes.cast(ptrs, _fpp),
                               out.ctypes.data_as(_f64p))
    if rc != 0:
        raise ValueError("oracle_add_dense failed: %d" % rc)
    del keep
    return out


def equation_dense(chains) -> np.ndarray:
    """A sum of chain products (mixed Add / Mul, Sec. 2 Operations): every addend by the dense
    definition of the chain product, added up in order.  chains: list of (dims, props, factors,
    trans or None)."""
    total = None
    for dims, props, factors, trans in chains:
        term = eval_dense(dims, props, factors, trans=trans)
        total = term if total is None else total + term
    return total


def equation_property(chains) -> int:
    """Property of the sum of the chains' products."""
    return sum_property([plan_bruteforce(d, p, trans=t)["result_prop"] for d, p, _, t in chains])
