"""ctypes binding of libmom.so: argument marshalling only.

Every function has the name of the C entry point it calls (include/mom.h).  PyTorch is used
for device memory and streams; all arithmetic happens in the library's HIP kernels.  There is
no fallback: if the library is not built, importing this module raises.
"""
import ctypes
import os
from typing import List, Optional, Sequence

import torch

from . import build as _build

MOM_GENERAL, MOM_LOWER_TRI, MOM_UPPER_TRI, MOM_IDENTITY, MOM_DIAGONAL = 0, 1, 2, 3, 4
MOM_OK = 0
MOM_OUT_ZERO_FILL_TRIANGLE = 1
MOM_MAX_FACTORS = 1024
MOM_STATIC_WORKSPACE_BYTES = 64 << 20

STATUS_NAMES = ["MOM_OK", "MOM_ERR_NULL", "MOM_ERR_BAD_N", "MOM_ERR_BAD_DIM", "MOM_ERR_BAD_PROP",
                "MOM_ERR_NOT_SQUARE", "MOM_ERR_OVERFLOW", "MOM_ERR_BAD_SPLITS", "MOM_ERR_WORKSPACE",
                "MOM_ERR_BUFFER_TOO_SMALL", "MOM_ERR_BAD_STRIDE", "MOM_ERR_UNSUPPORTED", "MOM_ERR_HIP",
                "MOM_ERR_NOMEM", "MOM_ERR_BAD_FLAGS", "MOM_ERR_NOT_READY", "MOM_ERR_BAD_TRANS"]

MOM_PLAN_MIN_MULTS, MOM_PLAN_MIN_TIME = 0, 1

EXPORTS = ["mom_chain_plan", "mom_plan_from_splits", "mom_chain_plan_ex", "mom_plan_destroy", "mom_plan_cost_mults", "mom_plan_cost_time_ps",
           "mom_plan_num_products", "mom_plan_result", "mom_plan_string", "mom_plan_splits",
           "mom_plan_product", "mom_plan_num_launches", "mom_plan_workspace_bytes", "mom_init", "mom_chain_eval", "mom_chain_eval_static", "mom_chain_eval_batched", "mom_equation_plan", "mom_equation_destroy", "mom_equation_result",
           "mom_equation_cost_mults", "mom_equation_workspace_bytes", "mom_equation_num_chains", "mom_equation_chain",
           "mom_equation_eval", "mom_probe_mfma_peak",
           "mom_status_string"]


class MomError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        name = STATUS_NAMES[status] if 0 <= status < len(STATUS_NAMES) else str(status)
        super().__init__("%s: %s (%s)" % (where, name, mom_status_string(status)))


def _load() -> ctypes.CDLL:
    if not _build.is_built():
        if os.environ.get("MOM_NO_AUTOBUILD"):
            raise ImportError("libmom.so is not built; run paper_2208_10391_amd/build.py")
        _build.build()
    return ctypes.CDLL(_build.LIB)


_lib = _load()
_i64p = ctypes.POINTER(ctypes.c_int64)
_i32p = ctypes.POINTER(ctypes.c_int32)
_vpp = ctypes.POINTER(ctypes.c_void_p)

_lib.mom_chain_plan.restype = ctypes.c_int
_lib.mom_chain_plan.argtypes = [_i64p, _i32p, ctypes.c_int32, _vpp]
_lib.mom_plan_from_splits.restype = ctypes.c_int
_lib.mom_plan_from_splits.argtypes = [_i64p, _i32p, ctypes.c_int32, _i32p, _vpp]
_lib.mom_chain_plan_ex.restype = ctypes.c_int
_lib.mom_chain_plan_ex.argtypes = [_i64p, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32, _i32p, _vpp]
_lib.mom_plan_destroy.restype = None
_lib.mom_plan_destroy.argtypes = [ctypes.c_void_p]
_lib.mom_plan_cost_mults.restype = ctypes.c_uint64
_lib.mom_plan_cost_mults.argtypes = [ctypes.c_void_p]
_lib.mom_plan_cost_time_ps.restype = ctypes.c_uint64
_lib.mom_plan_cost_time_ps.argtypes = [ctypes.c_void_p]
_lib.mom_plan_num_products.restype = ctypes.c_int32
_lib.mom_plan_num_products.argtypes = [ctypes.c_void_p]
_lib.mom_plan_result.restype = ctypes.c_int
_lib.mom_plan_result.argtypes = [ctypes.c_void_p, _i64p, _i64p, _i32p]
_lib.mom_plan_string.restype = ctypes.c_int
_lib.mom_plan_string.argtypes = [ctypes.c_void_p, ctypes.c_char_p, ctypes.c_size_t]
_lib.mom_plan_splits.restype = ctypes.c_int
_lib.mom_plan_splits.argtypes = [ctypes.c_void_p, _i32p, ctypes.c_int32]
_lib.mom_plan_product.restype = ctypes.c_int
_lib.mom_plan_product.argtypes = [ctypes.c_void_p, ctypes.c_int32, _i64p, _i32p, ctypes.POINTER(ctypes.c_uint64), _i32p]
_lib.mom_plan_num_launches.restype = ctypes.c_int32
_lib.mom_plan_num_launches.argtypes = [ctypes.c_void_p]
_lib.mom_plan_workspace_bytes.restype = ctypes.c_size_t
_lib.mom_plan_workspace_bytes.argtypes = [ctypes.c_void_p]
_lib.mom_init.restype = ctypes.c_int
_lib.mom_init.argtypes = []
_lib.mom_chain_eval.restype = ctypes.c_int
_lib.mom_chain_eval.argtypes = [ctypes.c_void_p, _vpp, _i64p, ctypes.c_void_p, ctypes.c_int64,
                                ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_void_p]
_lib.mom_chain_eval_static.restype = ctypes.c_int
_lib.mom_chain_eval_static.argtypes = [ctypes.c_void_p, _vpp, _i64p, ctypes.c_void_p, ctypes.c_int64,
                                       ctypes.c_uint32, ctypes.c_void_p]
_lib.mom_chain_eval_batched.restype = ctypes.c_int
_lib.mom_chain_eval_batched.argtypes = [ctypes.c_void_p, _vpp, _i64p, ctypes.c_void_p, ctypes.c_int64,
                                        ctypes.c_int32, ctypes.c_void_p]
_lib.mom_equation_plan.restype = ctypes.c_int
_lib.mom_equation_plan.argtypes = [_i64p, _i32p, _i32p, _i32p, ctypes.c_int32, ctypes.c_int32, _vpp]
_lib.mom_equation_destroy.restype = None
_lib.mom_equation_destroy.argtypes = [ctypes.c_void_p]
_lib.mom_equation_result.restype = ctypes.c_int
_lib.mom_equation_result.argtypes = [ctypes.c_void_p, _i64p, _i64p, _i32p]
_lib.mom_equation_cost_mults.restype = ctypes.c_uint64
_lib.mom_equation_cost_mults.argtypes = [ctypes.c_void_p]
_lib.mom_equation_workspace_bytes.restype = ctypes.c_size_t
_lib.mom_equation_workspace_bytes.argtypes = [ctypes.c_void_p]
_lib.mom_equation_num_chains.restype = ctypes.c_int32
_lib.mom_equation_num_chains.argtypes = [ctypes.c_void_p]
_lib.mom_equation_chain.restype = ctypes.c_void_p
_lib.mom_equation_chain.argtypes = [ctypes.c_void_p, ctypes.c_int32]
_lib.mom_equation_eval.restype = ctypes.c_int
_lib.mom_equation_eval.argtypes = [ctypes.c_void_p, _vpp, _i64p, ctypes.c_void_p, ctypes.c_int64,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_uint32, ctypes.c_void_p]
_lib.mom_probe_mfma_peak.restype = ctypes.c_int
_lib.mom_probe_mfma_peak.argtypes = [ctypes.c_int32, ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.c_void_p]
_lib.mom_status_string.restype = ctypes.c_char_p
_lib.mom_status_string.argtypes = [ctypes.c_int]


def library() -> ctypes.CDLL:
    return _lib


def mom_status_string(status: int) -> str:
    return _lib.mom_status_string(int(status)).decode()


class Plan:
    """Owner of a mom_plan_t handle."""

    def __init__(self, handle: int, dims: Sequence[int], props: Sequence[int], trans: Optional[Sequence[int]] = None):
        self.handle = ctypes.c_void_p(handle)
        self.dims = [int(d) for d in dims]
        self.props = [int(p) for p in props]
        self.trans = [0] * len(self.props) if trans is None else [1 if t else 0 for t in trans]

    def stored_shape(self, t: int):
        """Shape of factor t's buffer: the transpose's shape when the factor enters transposed."""
        r, c = self.dims[t], self.dims[t + 1]
        return (c, r) if self.trans[t] else (r, c)

    def __del__(self):
        if getattr(self, "handle", None):
            _lib.mom_plan_destroy(self.handle)
            self.handle = None

    @property
    def n(self) -> int:
        return len(self.props)

    @property
    def cost_mults(self) -> int:
        return mom_plan_cost_mults(self)

    @property
    def cost_time_ps(self) -> int:
        return int(_lib.mom_plan_cost_time_ps(self.handle))

    @property
    def string(self) -> str:
        return mom_plan_string(self)

    @property
    def splits(self) -> List[int]:
        return mom_plan_splits(self)

    @property
    def workspace_bytes(self) -> int:
        return mom_plan_workspace_bytes(self)

    @property
    def result(self):
        return mom_plan_result(self)


def _i64(values) -> ctypes.Array:
    return (ctypes.c_int64 * len(values))(*[int(v) for v in values])


def _i32(values) -> ctypes.Array:
    return (ctypes.c_int32 * max(len(values), 1))(*[int(v) for v in values])


def mom_chain_plan_ex(dims: Sequence[int], props: Sequence[int], trans: Optional[Sequence[int]] = None,
                      objective: int = MOM_PLAN_MIN_MULTS, preorder_splits: Optional[Sequence[int]] = None) -> Plan:
    """The general planning call: transposed factors (props are those of the STORED matrices),
    the objective, and optionally a forced tree."""
    n = len(props)
    if len(dims) != n + 1:
        raise ValueError("dims must have len(props)+1 entries")
    if trans is not None and len(trans) != n:
        raise ValueError("trans must have len(props) entries")
    if preorder_splits is not None:
        survivors = sum(1 for p in props if p != MOM_IDENTITY)
        if len(preorder_splits) != max(survivors - 1, 0):
            raise MomError(7, "mom_chain_plan_ex")
    out = ctypes.c_void_p()
    st = _lib.mom_chain_plan_ex(_i64(dims), _i32(props), None if trans is None else _i32(trans), n, int(objective),
                                None if preorder_splits is None else _i32(preorder_splits), ctypes.byref(out))
    if st != MOM_OK:
        raise MomError(st, "mom_chain_plan_ex")
    return Plan(out.value, dims, props, trans)


def mom_chain_plan(dims: Sequence[int], props: Sequence[int], trans: Optional[Sequence[int]] = None) -> Plan:
    if trans is not None:
        return mom_chain_plan_ex(dims, props, trans)
    n = len(props)
    if len(dims) != n + 1:
        raise ValueError("dims must have len(props)+1 entries")
    out = ctypes.c_void_p()
    st = _lib.mom_chain_plan(_i64(dims), _i32(props), n, ctypes.byref(out))
    if st != MOM_OK:
        raise MomError(st, "mom_chain_plan")
    return Plan(out.value, dims, props)


def mom_plan_from_splits(dims: Sequence[int], props: Sequence[int], preorder_splits: Sequence[int],
                         trans: Optional[Sequence[int]] = None) -> Plan:
    if trans is not None:
        return mom_chain_plan_ex(dims, props, trans, preorder_splits=preorder_splits)
    n = len(props)
    if len(dims) != n + 1:
        raise ValueError("dims must have len(props)+1 entries")
    survivors = sum(1 for p in props if p != MOM_IDENTITY)
    if len(preorder_splits) != max(survivors - 1, 0):
        raise MomError(7, "mom_plan_from_splits")
    out = ctypes.c_void_p()
    st = _lib.mom_plan_from_splits(_i64(dims), _i32(props), n, _i32(preorder_splits), ctypes.byref(out))
    if st != MOM_OK:
        raise MomError(st, "mom_plan_from_splits")
    return Plan(out.value, dims, props)


def mom_plan_cost_mults(plan: Plan) -> int:
    return int(_lib.mom_plan_cost_mults(plan.handle))


def mom_plan_num_products(plan: Plan) -> int:
    return int(_lib.mom_plan_num_products(plan.handle))


def mom_plan_result(plan: Plan):
    r, c, p = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
    st = _lib.mom_plan_result(plan.handle, ctypes.byref(r), ctypes.byref(c), ctypes.byref(p))
    if st != MOM_OK:
        raise MomError(st, "mom_plan_result")
    return int(r.value), int(c.value), int(p.value)


def mom_plan_string(plan: Plan) -> str:
    buf = ctypes.create_string_buffer(16 * plan.n + 16)
    st = _lib.mom_plan_string(plan.handle, buf, len(buf))
    if st != MOM_OK:
        raise MomError(st, "mom_plan_string")
    return buf.value.decode()


def mom_plan_splits(plan: Plan) -> List[int]:
    k = mom_plan_num_products(plan)
    out = (ctypes.c_int32 * max(k, 1))()
    st = _lib.mom_plan_splits(plan.handle, out, k)
    if st != MOM_OK:
        raise MomError(st, "mom_plan_splits")
    return [int(out[i]) for i in range(k)]


def mom_plan_product(plan: Plan, i: int) -> dict:
    """The i-th binary product in evaluation order: shape (m, k, n), props (left, right, result),
    mults, level."""
    shape, props = (ctypes.c_int64 * 3)(), (ctypes.c_int32 * 3)()
    mults, level = ctypes.c_uint64(), ctypes.c_int32()
    st = _lib.mom_plan_product(plan.handle, int(i), shape, props, ctypes.byref(mults), ctypes.byref(level))
    if st != MOM_OK:
        raise MomError(st, "mom_plan_product")
    return {"shape": tuple(int(x) for x in shape), "props": tuple(int(x) for x in props),
            "mults": int(mults.value), "level": int(level.value)}


def mom_plan_num_launches(plan: Plan) -> int:
    return int(_lib.mom_plan_num_launches(plan.handle))


def mom_plan_workspace_bytes(plan: Plan) -> int:
    return int(_lib.mom_plan_workspace_bytes(plan.handle))


def mom_init() -> None:
    """One-time set-up of the current device (needed before a FIRST evaluation is captured)."""
    st = _lib.mom_init()
    if st != MOM_OK:
        raise MomError(st, "mom_init")


def _stream_handle(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_factor(t: torch.Tensor, what: str):
    if not t.is_cuda or t.dtype != torch.float32:
        raise TypeError("%s must be a float32 tensor on the GPU" % what)


class BoundEval:
    """The marshalled arguments of one mom_chain_eval / mom_chain_eval_batched call, kept so that
    the same evaluation can be enqueued again without marshalling again (a launch-bound caller
    pays microseconds per call otherwise).  Holds references to every tensor it points into."""

    def __init__(self, entry, where: str, head: tuple, tail: tuple, out: torch.Tensor, keep: tuple):
        self._entry, self._where, self._head, self._tail = entry, where, head, tail
        self.out = out
        self._keep = keep

    def __call__(self, stream=None) -> torch.Tensor:
        st = self._entry(*self._head, _stream_handle(stream), *self._tail)
        if st != MOM_OK:
            raise MomError(st, self._where)
        return self.out


def bind_chain_eval(plan: Plan, factors: Sequence[Optional[torch.Tensor]], out: Optional[torch.Tensor] = None,
                    workspace: Optional[torch.Tensor] = None, flags: int = 0, static: bool = False) -> BoundEval:
    """Checks and marshals the arguments of mom_chain_eval; calling the result enqueues the plan
    on the (current) stream.  factors[t] is a 2-D f32 CUDA tensor with unit column stride (None
    for Identity factors); `out` and `workspace` are allocated with torch when not given (out is
    NOT cleared: a triangular result leaves its other half untouched unless flags has
    MOM_OUT_ZERO_FILL_TRIANGLE).  With static=True the call is mom_chain_eval_static: no workspace
    tensor at all, the library's own per-GPU array is used."""
    n = plan.n
    if len(factors) != n:
        raise ValueError("expected %d factors" % n)
    ptrs = (ctypes.c_void_p * n)()
    lds = (ctypes.c_int64 * n)()
    for t, f in enumerate(factors):
        if f is None:
            ptrs[t] = None
            lds[t] = plan.stored_shape(t)[1]
            continue
        _check_factor(f, "factor %d" % t)
        if f.dim() != 2 or tuple(f.shape) != plan.stored_shape(t) or f.stride(1) != 1:
            raise ValueError("factor %d must be %dx%d with unit column stride" % ((t,) + plan.stored_shape(t)))
        ptrs[t] = f.data_ptr()
        lds[t] = f.stride(0) if f.shape[0] > 1 else max(f.stride(0), f.shape[1])
    rows, cols, _ = mom_plan_result(plan)
    dev = next((f.device for f in factors if f is not None), torch.device("cuda", torch.cuda.current_device()))
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    _check_factor(out, "out")
    if tuple(out.shape) != (rows, cols) or out.stride(1) != 1:
        raise ValueError("out must be %dx%d with unit column stride" % (rows, cols))
    ld_out = out.stride(0) if rows > 1 else max(out.stride(0), cols)
    if static:
        head = (plan.handle, ctypes.cast(ptrs, _vpp), lds, ctypes.c_void_p(out.data_ptr()), ld_out, int(flags))
        return BoundEval(_lib.mom_chain_eval_static, "mom_chain_eval_static", head, (), out,
                         (plan, ptrs, lds, tuple(factors)))
    need = mom_plan_workspace_bytes(plan)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    head = (plan.handle, ctypes.cast(ptrs, _vpp), lds, ctypes.c_void_p(out.data_ptr()), ld_out,
            ctypes.c_void_p(ws_ptr), ws_bytes, int(flags))
    return BoundEval(_lib.mom_chain_eval, "mom_chain_eval", head, (), out,
                     (plan, ptrs, lds, tuple(factors), workspace))


def mom_chain_eval(plan: Plan, factors: Sequence[Optional[torch.Tensor]], out: Optional[torch.Tensor] = None,
                   workspace: Optional[torch.Tensor] = None, flags: int = 0, stream=None) -> torch.Tensor:
    """One call of the C entry point: marshal (bind_chain_eval) and enqueue."""
    return bind_chain_eval(plan, factors, out, workspace, flags)(stream)


def bind_chain_eval_batched(plan: Plan, factors: Sequence[Optional[torch.Tensor]],
                            out: Optional[torch.Tensor] = None) -> BoundEval:
    """Checks and marshals the arguments of mom_chain_eval_batched.  factors[t]: [batch, dims[t],
    dims[t+1]] f32 CUDA tensor whose matrices are packed (None for Identity factors).  One kernel
    launch for the whole batch."""
    n = plan.n
    if len(factors) != n:
        raise ValueError("expected %d factors" % n)
    batch = next((f.shape[0] for f in factors if f is not None), None)
    if batch is None and out is None:
        raise ValueError("an all-Identity batched chain needs an explicit `out` to give the batch size")
    ptrs = (ctypes.c_void_p * n)()
    strides = (ctypes.c_int64 * n)()
    for t, f in enumerate(factors):
        if f is None:
            ptrs[t] = None
            strides[t] = plan.dims[t] * plan.dims[t + 1]
            continue
        _check_factor(f, "factor %d" % t)
        r, c = plan.stored_shape(t)
        if f.dim() != 3 or tuple(f.shape[1:]) != (r, c) or f.shape[0] != batch:
            raise ValueError("factor %d must be [batch, %d, %d]" % (t, r, c))
        if f.stride(2) != 1 or (r > 1 and f.stride(1) != c):
            raise ValueError("factor %d: matrices must be packed row-major" % t)
        ptrs[t] = f.data_ptr()
        strides[t] = f.stride(0) if batch > 1 else max(f.stride(0), r * c)
    rows, cols, _ = mom_plan_result(plan)
    if batch is None:
        batch = out.shape[0]
    dev = next((f.device for f in factors if f is not None), out.device if out is not None else None)
    if out is None:
        out = torch.empty((batch, rows, cols), dtype=torch.float32, device=dev)
    _check_factor(out, "out")
    if tuple(out.shape) != (batch, rows, cols) or not out[0].is_contiguous():
        raise ValueError("out must be [batch, %d, %d] with packed matrices" % (rows, cols))
    out_stride = out.stride(0) if batch > 1 else max(out.stride(0), rows * cols)
    head = (plan.handle, ctypes.cast(ptrs, _vpp), strides, ctypes.c_void_p(out.data_ptr()), out_stride, batch)
    return BoundEval(_lib.mom_chain_eval_batched, "mom_chain_eval_batched", head, (), out,
                     (plan, ptrs, strides, tuple(factors)))


def mom_chain_eval_static(plan: Plan, factors: Sequence[Optional[torch.Tensor]], out: Optional[torch.Tensor] = None,
                          flags: int = 0, stream=None) -> torch.Tensor:
    """One call of the C entry point that uses the library's own per-GPU workspace (the output
    tensor, when not given, is still allocated here, by torch, before the call)."""
    return bind_chain_eval(plan, factors, out, None, flags, static=True)(stream)


def mom_chain_eval_batched(plan: Plan, factors: Sequence[Optional[torch.Tensor]],
                           out: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """One call of the C entry point: marshal (bind_chain_eval_batched) and enqueue."""
    return bind_chain_eval_batched(plan, factors, out)(stream)


class Equation:
    """Owner of a mom_equation_t handle: a sum of chains.  chains: list of (dims, props, trans or None)."""

    def __init__(self, handle: int, chains):
        self.handle = ctypes.c_void_p(handle)
        self.chains = [([int(d) for d in dims], [int(p) for p in props],
                        [0] * len(props) if trans is None else [1 if t else 0 for t in trans])
                       for dims, props, trans in chains]

    def __del__(self):
        if getattr(self, "handle", None):
            _lib.mom_equation_destroy(self.handle)
            self.handle = None

    @property
    def result(self):
        r, c, p = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        st = _lib.mom_equation_result(self.handle, ctypes.byref(r), ctypes.byref(c), ctypes.byref(p))
        if st != MOM_OK:
            raise MomError(st, "mom_equation_result")
        return int(r.value), int(c.value), int(p.value)

    @property
    def cost_mults(self) -> int:
        return int(_lib.mom_equation_cost_mults(self.handle))

    @property
    def workspace_bytes(self) -> int:
        return int(_lib.mom_equation_workspace_bytes(self.handle))

    def chain_string(self, c: int) -> str:
        """Parenthesisation of addend c."""
        h = _lib.mom_equation_chain(self.handle, int(c))
        buf = ctypes.create_string_buffer(16 * len(self.chains[c][1]) + 16)
        st = _lib.mom_plan_string(ctypes.c_void_p(h), buf, len(buf))
        if st != MOM_OK:
            raise MomError(st, "mom_plan_string")
        return buf.value.decode()


def mom_equation_plan(chains, objective: int = MOM_PLAN_MIN_MULTS) -> Equation:
    """chains: list of (dims, props, trans or None), every chain with the same rows x cols."""
    dims, props, trans, lens = [], [], [], []
    any_trans = any(t is not None for _, _, t in chains)
    for d, p, t in chains:
        if len(d) != len(p) + 1:
            raise ValueError("dims must have len(props)+1 entries")
        dims += list(d)
        props += list(p)
        trans += [0] * len(p) if t is None else list(t)
        lens.append(len(p))
    out = ctypes.c_void_p()
    st = _lib.mom_equation_plan(_i64(dims), _i32(props), _i32(trans) if any_trans else None, _i32(lens), len(lens),
                                int(objective), ctypes.byref(out))
    if st != MOM_OK:
        raise MomError(st, "mom_equation_plan")
    return Equation(out.value, chains)


def bind_equation_eval(eq: Equation, factors: Sequence[Sequence[Optional[torch.Tensor]]], out: Optional[torch.Tensor] = None,
                       workspace: Optional[torch.Tensor] = None, flags: int = 0) -> BoundEval:
    """Checks and marshals the arguments of mom_equation_eval; calling the result enqueues the
    equation on the (current) stream.  factors[c][t]: the buffer of factor t of addend c (None
    for Identity), stored shape."""
    flat, stored = [], []
    for (dims, props, trans), fs in zip(eq.chains, factors):
        if len(fs) != len(props):
            raise ValueError("wrong number of factors in an addend")
        for t, f in enumerate(fs):
            r, c = (dims[t + 1], dims[t]) if trans[t] else (dims[t], dims[t + 1])
            flat.append(f)
            stored.append((r, c))
    n = len(flat)
    ptrs = (ctypes.c_void_p * n)()
    lds = (ctypes.c_int64 * n)()
    for i, (f, (r, c)) in enumerate(zip(flat, stored)):
        if f is None:
            ptrs[i] = None
            lds[i] = c
            continue
        _check_factor(f, "factor %d" % i)
        if f.dim() != 2 or tuple(f.shape) != (r, c) or f.stride(1) != 1:
            raise ValueError("factor %d must be %dx%d with unit column stride" % (i, r, c))
        ptrs[i] = f.data_ptr()
        lds[i] = f.stride(0) if r > 1 else max(f.stride(0), c)
    rows, cols, _ = eq.result
    dev = next((f.device for f in flat if f is not None), torch.device("cuda", torch.cuda.current_device()))
    if out is None:
        out = torch.empty((rows, cols), dtype=torch.float32, device=dev)
    _check_factor(out, "out")
    if tuple(out.shape) != (rows, cols) or out.stride(1) != 1:
        raise ValueError("out must be %dx%d with unit column stride" % (rows, cols))
    need = eq.workspace_bytes
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    ld_out = out.stride(0) if rows > 1 else max(out.stride(0), cols)
    head = (eq.handle, ctypes.cast(ptrs, _vpp), lds, ctypes.c_void_p(out.data_ptr()), ld_out,
            ctypes.c_void_p(ws_ptr), ws_bytes, int(flags))
    return BoundEval(_lib.mom_equation_eval, "mom_equation_eval", head, (), out, (eq, ptrs, lds, tuple(flat), workspace))


def mom_equation_eval(eq: Equation, factors: Sequence[Sequence[Optional[torch.Tensor]]], out: Optional[torch.Tensor] = None,
                      workspace: Optional[torch.Tensor] = None, flags: int = 0, stream=None) -> torch.Tensor:
    """One call of the C entry point: marshal (bind_equation_eval) and enqueue."""
    return bind_equation_eval(eq, factors, out, workspace, flags)(stream)


def mom_probe_mfma_peak(iters: int, sink: torch.Tensor, stream=None) -> float:
    """Enqueue one launch of the register-only MFMA loop; returns its floating-point operations.
    `sink`: a CUDA tensor of at least 1024 bytes.  The caller times the launch."""
    if not sink.is_cuda or sink.numel() * sink.element_size() < 1024:
        raise ValueError("sink must be a GPU tensor of at least 1024 bytes")
    flop = ctypes.c_double(0.0)
    st = _lib.mom_probe_mfma_peak(int(iters), ctypes.c_void_p(sink.data_ptr()), ctypes.byref(flop), _stream_handle(stream))
    if st != MOM_OK:
        raise MomError(st, "mom_probe_mfma_peak")
    return flop.value
