"""Thin ctypes binding of libewf.so: the same names as the C ABI in include/ewf.h, argument
marshalling only.  Every step of the computation runs in the library's HIP kernels; there is
no fallback: importing this module fails if the library has not been built.

Tensors are anything with ``data_ptr()``, ``shape`` and ``stride()`` (PyTorch tensors on the
GPU), or a ``TensorRef`` for host-only planning tests.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# EWF_LIBRARY names another build of the same library (the host-sanitizer build, say)
LIB_PATH = os.environ.get("EWF_LIBRARY") or os.path.join(_HERE, "libewf.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1605_02688_amd.build`")
# PyTorch ships a HIP runtime of its own.  The dynamic loader keeps one runtime per process, the
# first one loaded; device memory handed over by PyTorch is only valid in PyTorch's.  So when
# PyTorch is installed it is imported before the library (a process that never uses PyTorch
# simply gets the system runtime).
try:
    import torch  # noqa: F401
except ImportError:
    pass
_lib = ctypes.CDLL(LIB_PATH)

MAX_DIMS = 8
OK = 0
EINVAL, ETYPE, ESHAPE, EALIAS, ECOMPILE, EHIP, ENOMEM, EUNSUPPORTED = -1, -2, -3, -4, -5, -6, -7, -8
F32, F16, I32 = 0, 1, 2
DTYPES = {"f32": F32, "f16": F16, "i32": I32}
OPS = {name: i for i, name in enumerate(
    ["add", "sub", "mul", "div", "neg", "abs", "exp", "log", "log1p", "sqrt", "tanh", "sigmoid", "max", "min",
     "pow", "where", "gt", "ge", "lt", "le", "eq", "ne", "expm1", "sqr", "recip"])}
REDOPS = {"sum": 0, "max": 1, "min": 2, "prod": 3, "argmax": 4}
KERNEL_CLASSES = {0: "none", 1: "tile", 2: "tile_reduce", 3: "row", 4: "col", 5: "multi", 6: "lane"}


class EwfError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ewf status {status}: {message}")
        self.status = status
        self.message = message


class ewf_options(ctypes.Structure):
    _fields_ = [("math_mode", ctypes.c_int32), ("force_scalar", ctypes.c_int32),
                ("force_index64", ctypes.c_int32), ("block_threads", ctypes.c_int32),
                ("unroll", ctypes.c_int32), ("max_blocks", ctypes.c_int32),
                ("no_lds_staging", ctypes.c_int32), ("streaming", ctypes.c_int32),
                ("tile_elems", ctypes.c_int32), ("waves_per_simd", ctypes.c_int32),
                ("no_prefetch", ctypes.c_int32), ("xcd_remap", ctypes.c_int32),
                ("no_rewrite", ctypes.c_int32), ("split_rows", ctypes.c_int32),
                ("plain_extremes", ctypes.c_int32), ("reserved", ctypes.c_int32 * 1)]


class ewf_tensor(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("shape", ctypes.POINTER(ctypes.c_int64)),
                ("strides", ctypes.POINTER(ctypes.c_int64))]


class ewf_call(ctypes.Structure):
    _fields_ = [("exec", ctypes.c_void_p), ("tin", ctypes.POINTER(ewf_tensor)), ("tout", ctypes.POINTER(ewf_tensor)),
                ("scalars", ctypes.POINTER(ctypes.c_double)), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("hip_stream", ctypes.c_void_p),
                ("nin", ctypes.c_int32), ("nout", ctypes.c_int32), ("nscalars", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class ewf_plan_info(ctypes.Structure):
    _fields_ = [("kernel_class", ctypes.c_int32), ("rank", ctypes.c_int32),
                ("extent", ctypes.c_int64 * MAX_DIMS), ("reduced", ctypes.c_int32 * MAX_DIMS),
                ("vec", ctypes.c_int32), ("index_bits", ctypes.c_int32), ("noperands", ctypes.c_int32),
                ("block_threads", ctypes.c_int32), ("grid_blocks", ctypes.c_int32),
                ("lds_bytes", ctypes.c_int32), ("staged_operands", ctypes.c_int32),
                ("tile", ctypes.c_int64 * MAX_DIMS)]


class ewf_node_info(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("op", ctypes.c_int32), ("nargs", ctypes.c_int32),
                ("args", ctypes.c_int32 * 3), ("index", ctypes.c_int32), ("axes", ctypes.c_uint32),
                ("keep", ctypes.c_int32), ("vtype", ctypes.c_int32), ("storage", ctypes.c_int32),
                ("bcast", ctypes.c_uint32), ("cval", ctypes.c_double)]


_vp = ctypes.c_void_p
_i32 = ctypes.c_int32
_sigs = {
    "ewf_graph_create": (_i32, [_i32, ctypes.POINTER(_vp)]),
    "ewf_graph_destroy": (None, [_vp]),
    "ewf_input": (_i32, [_vp, _i32, ctypes.POINTER(ctypes.c_uint8)]),
    "ewf_scalar": (_i32, [_vp, _i32]),
    "ewf_const": (_i32, [_vp, _i32, ctypes.c_double]),
    "ewf_iota": (_i32, [_vp, _i32]),
    "ewf_apply": (_i32, [_vp, _i32, ctypes.POINTER(_i32), _i32]),
    "ewf_cast": (_i32, [_vp, _i32, _i32]),
    "ewf_reduce": (_i32, [_vp, _i32, _i32, ctypes.POINTER(_i32), _i32, _i32]),
    "ewf_output": (_i32, [_vp, _i32, _i32]),
    "ewf_grad": (_i32, [_vp, ctypes.POINTER(_i32), ctypes.POINTER(_i32), _i32, ctypes.POINTER(_i32), _i32,
                        ctypes.POINTER(_i32)]),
    "ewf_compile": (_i32, [_vp, ctypes.POINTER(ewf_options), ctypes.POINTER(_vp)]),
    "ewf_exec_destroy": (None, [_vp]),
    "ewf_output_shape": (_i32, [_vp, ctypes.POINTER(ewf_tensor), _i32, _i32, ctypes.POINTER(_i32),
                                ctypes.POINTER(ctypes.c_int64)]),
    "ewf_plan": (_i32, [_vp, ctypes.POINTER(ewf_tensor), _i32, ctypes.POINTER(ewf_tensor), _i32,
                        ctypes.POINTER(ctypes.c_size_t)]),
    "ewf_workspace_init": (_i32, [_vp, ctypes.c_size_t, _vp]),
    "ewf_run": (_i32, [_vp, ctypes.POINTER(ewf_tensor), _i32, ctypes.POINTER(ctypes.c_double), _i32,
                       ctypes.POINTER(ewf_tensor), _i32, _vp, ctypes.c_size_t, _vp]),
    "ewf_run_static": (_i32, [_vp, ctypes.POINTER(ewf_tensor), _i32, ctypes.POINTER(ctypes.c_double), _i32,
                              ctypes.POINTER(ewf_tensor), _i32, _vp]),
    "ewf_run_call": (_i32, [ctypes.POINTER(ewf_call)]),
    "ewf_run_sequence": (_i32, [ctypes.POINTER(ewf_call), _i32, ctypes.POINTER(_i32)]),
    "ewf_last_error": (ctypes.c_char_p, []),
    "ewf_debug_graph_count": (_i32, [_vp]),
    "ewf_debug_graph_node": (_i32, [_vp, _i32, ctypes.POINTER(ewf_node_info)]),
    "ewf_debug_plan_info": (_i32, [_vp, ctypes.POINTER(ewf_plan_info)]),
    "ewf_debug_operand_strides": (_i32, [_vp, _i32, ctypes.POINTER(ctypes.c_int64)]),
    "ewf_debug_source": (ctypes.c_char_p, [_vp]),
    "ewf_debug_stage_plan_info": (_i32, [_vp, _i32, ctypes.POINTER(ewf_plan_info)]),
    "ewf_debug_stage_source": (ctypes.c_char_p, [_vp, _i32]),
    "ewf_debug_compile_count": (_i32, [_vp]),
    "ewf_debug_graph_size": (_i32, [_vp, ctypes.POINTER(_i32), ctypes.POINTER(_i32)]),
    "ewf_copy_bytes": (_i32, [_vp, _vp, ctypes.c_size_t, _vp]),
    "ewf_debug_peak_concurrent_compiles": (_i32, [ctypes.POINTER(_i32)]),
    "ewf_debug_inject_fault": (_i32, [_i32, _i32]),
    "ewf_debug_time_kernels": (_i32, [_vp, _i32]),
    "ewf_debug_kernel_times": (_i32, [_vp, ctypes.POINTER(ctypes.c_float), _i32, ctypes.POINTER(_i32)]),
    "ewf_set_cache_dir": (_i32, [ctypes.c_char_p]),
    "ewf_debug_cache_stats": (_i32, [ctypes.POINTER(_i32), ctypes.POINTER(_i32), ctypes.POINTER(_i32)]),
}
for _name, (_res, _args) in _sigs.items():
    _f = getattr(_lib, _name)
    _f.restype = _res
    _f.argtypes = _args

EXPORTED = tuple(_sigs)


def last_error() -> str:
    return _lib.ewf_last_error().decode(errors="replace")


def _check(st: int) -> int:
    if st < 0:
        raise EwfError(st, last_error())
    return st


# ------------------------------------------------------------------ C ABI, one to one

def graph_create(ndim: int) -> int:
    g = _vp()
    _check(_lib.ewf_graph_create(ndim, ctypes.byref(g)))
    return g.value


def graph_destroy(g: int) -> None:
    _lib.ewf_graph_destroy(g)


def input(g: int, storage: int, bcast: Sequence[bool]) -> int:  # noqa: A001 (mirrors ewf_input)
    flags = (ctypes.c_uint8 * max(1, len(bcast)))(*[1 if b else 0 for b in bcast])
    return _check(_lib.ewf_input(g, storage, flags))


def scalar(g: int, dtype: int) -> int:
    return _check(_lib.ewf_scalar(g, dtype))


def const(g: int, dtype: int, value: float) -> int:
    return _check(_lib.ewf_const(g, dtype, float(value)))


def iota(g: int, axis: int) -> int:
    return _check(_lib.ewf_iota(g, axis))


def apply(g: int, op: int, args: Sequence[int]) -> int:
    a = (_i32 * max(1, len(args)))(*args)
    return _check(_lib.ewf_apply(g, op, a, len(args)))


def cast(g: int, v: int, to: int) -> int:
    return _check(_lib.ewf_cast(g, v, to))


def reduce(g: int, redop: int, v: int, axes: Sequence[int], keep_as_bcast: bool) -> int:
    a = (_i32 * max(1, len(axes)))(*axes)
    return _check(_lib.ewf_reduce(g, redop, v, a, len(axes), 1 if keep_as_bcast else 0))


def grad(g: int, ys: Sequence[int], ybars: Sequence[int], wrt: Sequence[int]) -> List[int]:
    ya = (_i32 * len(ys))(*ys)
    yb = (_i32 * len(ybars))(*ybars)
    wa = (_i32 * len(wrt))(*wrt)
    out = (_i32 * len(wrt))()
    _check(_lib.ewf_grad(g, ya, yb, len(ys), wa, len(wrt), out))
    return list(out)


def output(g: int, v: int, storage: int) -> None:
    _check(_lib.ewf_output(g, v, storage))


def compile(g: int, options: Optional[ewf_options] = None) -> int:  # noqa: A001
    e = _vp()
    _check(_lib.ewf_compile(g, ctypes.byref(options) if options is not None else None, ctypes.byref(e)))
    return e.value


def exec_destroy(e: int) -> None:
    _lib.ewf_exec_destroy(e)


@dataclass
class TensorRef:
    """A pointer + shape + element strides, for planning without device memory."""
    ptr: int
    shape: Tuple[int, ...]
    strides: Tuple[int, ...]

    def data_ptr(self) -> int:
        return self.ptr

    def stride(self) -> Tuple[int, ...]:
        return self.strides


def _marshal(tensors: Sequence) -> Tuple[ctypes.Array, list]:
    arr = (ewf_tensor * max(1, len(tensors)))()
    keep = []
    for k, t in enumerate(tensors):
        shape = tuple(int(x) for x in t.shape)
        strides = tuple(int(x) for x in t.stride())
        sh = (ctypes.c_int64 * max(1, len(shape)))(*shape)
        st = (ctypes.c_int64 * max(1, len(strides)))(*strides)
        keep += [sh, st]
        arr[k].ptr = t.data_ptr()
        arr[k].shape = sh
        arr[k].strides = st
    return arr, keep


def output_shape(e: int, inputs: Sequence, k: int) -> Tuple[int, ...]:
    tin, _keep = _marshal(inputs)
    rank = _i32()
    shape = (ctypes.c_int64 * MAX_DIMS)()
    _check(_lib.ewf_output_shape(e, tin, len(inputs), k, ctypes.byref(rank), shape))
    return tuple(shape[d] for d in range(rank.value))


def plan(e: int, inputs: Sequence, outputs: Sequence) -> int:
    tin, _k1 = _marshal(inputs)
    tout, _k2 = _marshal(outputs)
    ws = ctypes.c_size_t()
    _check(_lib.ewf_plan(e, tin, len(inputs), tout, len(outputs), ctypes.byref(ws)))
    return ws.value


def workspace_init(ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.ewf_workspace_init(ptr, nbytes, stream))


def run(e: int, inputs: Sequence, scalars: Sequence[float], outputs: Sequence, workspace_ptr: int = 0,
        workspace_bytes: int = 0, stream: int = 0) -> None:
    tin, _k1 = _marshal(inputs)
    tout, _k2 = _marshal(outputs)
    sc = (ctypes.c_double * max(1, len(scalars)))(*[float(s) for s in scalars])
    _check(_lib.ewf_run(e, tin, len(inputs), sc, len(scalars), tout, len(outputs), workspace_ptr or None,
                        workspace_bytes, stream or None))


STATIC_WORKSPACE_BYTES = 4 << 20


def run_static(e: int, inputs: Sequence, scalars: Sequence[float], outputs: Sequence, stream: int = 0) -> None:
    tin, _k1 = _marshal(inputs)
    tout, _k2 = _marshal(outputs)
    sc = (ctypes.c_double * max(1, len(scalars)))(*[float(s) for s in scalars])
    _check(_lib.ewf_run_static(e, tin, len(inputs), sc, len(scalars), tout, len(outputs), stream or None))


def debug_plan_info(e: int, stage: int = -1) -> dict:
    """The last plan; with ``stage`` >= 0, that stage of a plan in several passes."""
    info = ewf_plan_info()
    if stage >= 0:
        _check(_lib.ewf_debug_stage_plan_info(e, stage, ctypes.byref(info)))
    else:
        _check(_lib.ewf_debug_plan_info(e, ctypes.byref(info)))
    r = info.rank
    return {"kernel_class": KERNEL_CLASSES.get(info.kernel_class, "?"), "rank": r,
            "extent": tuple(info.extent[d] for d in range(r)),
            "reduced": tuple(bool(info.reduced[d]) for d in range(r)),
            "tile": tuple(info.tile[d] for d in range(r)),
            "vec": info.vec, "index_bits": info.index_bits, "noperands": info.noperands,
            "block_threads": info.block_threads, "grid_blocks": info.grid_blocks,
            "lds_bytes": info.lds_bytes, "staged_operands": info.staged_operands}


def debug_operand_strides(e: int, k: int, rank: int) -> Tuple[int, ...]:
    st = (ctypes.c_int64 * MAX_DIMS)()
    _check(_lib.ewf_debug_operand_strides(e, k, st))
    return tuple(st[d] for d in range(rank))


def debug_source(e: int, stage: int = -1) -> str:
    if stage >= 0:
        return _lib.ewf_debug_stage_source(e, stage).decode()
    return _lib.ewf_debug_source(e).decode()


def debug_compile_count(e: int) -> int:
    return _lib.ewf_debug_compile_count(e)


def debug_graph_size(e: int) -> Tuple[int, int]:
    a, b = _i32(), _i32()
    _check(_lib.ewf_debug_graph_size(e, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def set_cache_dir(path: Optional[str]) -> None:
    _check(_lib.ewf_set_cache_dir(path.encode() if path else None))


def debug_cache_stats() -> dict:
    a, b, c = _i32(), _i32(), _i32()
    _check(_lib.ewf_debug_cache_stats(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return {"memory_hits": a.value, "disk_hits": b.value, "compiles": c.value}


def debug_peak_concurrent_compiles() -> int:
    n = _i32(0)
    _check(_lib.ewf_debug_peak_concurrent_compiles(ctypes.byref(n)))
    return n.value


def debug_inject_fault(kind: int, after: int = 0) -> None:
    _check(_lib.ewf_debug_inject_fault(kind, after))


def debug_time_kernels(e: int, slots: int) -> None:
    _check(_lib.ewf_debug_time_kernels(e, slots))


def debug_kernel_times(e: int, capacity: int) -> List[float]:
    """Durations in milliseconds of the main kernels launched since timing was turned on."""
    ms = (ctypes.c_float * max(1, capacity))()
    n = _i32(0)
    _check(_lib.ewf_debug_kernel_times(e, ms, capacity, ctypes.byref(n)))
    return [float(ms[i]) for i in range(n.value)]


def copy_bytes(dst_ptr: int, src_ptr: int, nbytes: int, stream: int = 0) -> None:
    _check(_lib.ewf_copy_bytes(dst_ptr, src_ptr, nbytes, stream or None))


# ------------------------------------------------------------------ convenience

def options(**kw) -> ewf_options:
    o = ewf_options()
    for k, v in kw.items():
        setattr(o, k, int(v))
    return o


def build_graph(spec, return_ids: bool = False):
    """Replays a data-only graph description (``ndim``, ``nodes``, ``outputs``; node tuples as
    produced by ``workloads.GraphSpec``) through the graph-building calls."""
    g = graph_create(spec.ndim)
    try:
        ids: List[int] = []
        grad_results = {}
        for node in spec.nodes:
            kind = node[0]
            if kind == "input":
                ids.append(input(g, DTYPES[node[2]], node[3]))
            elif kind == "scalar":
                ids.append(scalar(g, DTYPES[node[2]]))
            elif kind == "const":
                ids.append(const(g, DTYPES[node[1]], node[2]))
            elif kind == "iota":
                ids.append(iota(g, node[1]))
            elif kind == "apply":
                ids.append(apply(g, OPS[node[1]], [ids[a] for a in node[2]]))
            elif kind == "cast":
                ids.append(cast(g, ids[node[1]], DTYPES[node[2]]))
            elif kind == "reduce":
                ids.append(reduce(g, REDOPS[node[1]], ids[node[2]], node[3], node[4]))
            elif kind == "grad":
                # one differentiation call; its results are picked up by "gradof" nodes
                grad_results[len(ids)] = grad(g, [ids[v] for v in node[1]], [ids[v] for v in node[2]], [ids[v] for v in node[3]])
                ids.append(-1)
            elif kind == "gradof":
                ids.append(grad_results[node[1]][node[2]])
            else:
                raise ValueError(kind)
        for v, storage in spec.outputs:
            output(g, ids[v], DTYPES[storage])
    except Exception:
        graph_destroy(g)
        raise
    return (g, ids) if return_ids else g


def export_spec(spec):
    """Replays ``spec`` through the graph-building calls (differentiation requests included) and
    reads the resulting node list back as a plain description without such requests: what the
    library will compile, in a form any evaluator of descriptions can take."""
    from workloads import GraphSpec
    names = {v: k for k, v in OPS.items()}
    rnames = {v: k for k, v in REDOPS.items()}
    dnames = {v: k for k, v in DTYPES.items()}
    g, ids = build_graph(spec, return_ids=True)
    try:
        out = GraphSpec(spec.ndim)
        info = ewf_node_info()
        for i in range(_lib.ewf_debug_graph_count(g)):
            _check(_lib.ewf_debug_graph_node(g, i, ctypes.byref(info)))
            a = [info.args[k] for k in range(info.nargs)]
            bc = tuple(bool(info.bcast >> d & 1) for d in range(spec.ndim))
            if info.kind == 0:
                out.input(dnames[info.storage], bc)
            elif info.kind == 1:
                out.scalar(dnames[info.vtype])
            elif info.kind == 2:
                out.const(info.cval, dnames[info.vtype])
            elif info.kind == 3:
                out.iota(info.index)
            elif info.kind == 4:
                out.apply(names[info.op], *a)
            elif info.kind == 5:
                out.cast(a[0], dnames[info.op])
            else:
                out.reduce(rnames[info.op], a[0], [d for d in range(spec.ndim) if info.axes >> d & 1], bool(info.keep))
        for v, storage in spec.outputs:
            out.output(ids[v], storage)
        return out
    finally:
        graph_destroy(g)


class Expression:
    """compile once, run many times; owns the executable handle."""

    def __init__(self, spec, **opts):
        g = build_graph(spec)
        try:
            self.handle = compile(g, options(**opts) if opts else None)
        finally:
            graph_destroy(g)
        self.n_outputs = len(spec.outputs)

    def close(self) -> None:
        # at interpreter shutdown the module's globals may already be gone: then the process
        # is ending and the handle goes with it
        if getattr(self, "handle", None) and exec_destroy is not None:
            exec_destroy(self.handle)
            self.handle = None

    __del__ = close

    def output_shapes(self, inputs: Sequence) -> List[Tuple[int, ...]]:
        return [output_shape(self.handle, inputs, k) for k in range(self.n_outputs)]

    def plan(self, inputs: Sequence, outputs: Sequence) -> int:
        return plan(self.handle, inputs, outputs)

    def run(self, inputs, outputs, scalars=(), workspace=None, stream: int = 0) -> None:
        wptr = workspace.data_ptr() if workspace is not None else 0
        wbytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        run(self.handle, inputs, scalars, outputs, wptr, wbytes, stream)

    def run_static(self, inputs, outputs, scalars=(), stream: int = 0) -> None:
        """ewf_run_static: the library's static workspace, nothing set up or allocated by the call
        (the layout must have been planned with `plan`)."""
        run_static(self.handle, inputs, scalars, outputs, stream)

    def bind(self, inputs, outputs, scalars=(), workspace=None, stream: int = 0) -> "BoundCall":
        """Marshals the arguments once; ``BoundCall.launch()`` is then a single ewf_run call."""
        return BoundCall(self, inputs, outputs, scalars, workspace, stream)

    def info(self, stage: int = -1) -> dict:
        return debug_plan_info(self.handle, stage)

    def source(self, stage: int = -1) -> str:
        return debug_source(self.handle, stage)

    def graph_size(self) -> Tuple[int, int]:
        """(nodes described, nodes compiled after the rewrites)."""
        return debug_graph_size(self.handle)


class BoundCall:
    """ewf_run with its argument arrays prepared once (for launch loops: the Python-side
    marshalling otherwise costs more than a small kernel).  Keeps the tensors alive."""

    def __init__(self, expr: Expression, inputs, outputs, scalars=(), workspace=None, stream: int = 0):
        self.expr = expr
        self._tensors = (list(inputs), list(outputs), workspace)
        self._tin, self._k1 = _marshal(inputs)
        self._tout, self._k2 = _marshal(outputs)
        self._sc = (ctypes.c_double * max(1, len(scalars)))(*[float(s) for s in scalars])
        c = ewf_call()
        c.exec = expr.handle
        c.tin = ctypes.cast(self._tin, ctypes.POINTER(ewf_tensor))
        c.tout = ctypes.cast(self._tout, ctypes.POINTER(ewf_tensor))
        c.scalars = ctypes.cast(self._sc, ctypes.POINTER(ctypes.c_double))
        c.workspace = workspace.data_ptr() if workspace is not None else None
        c.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
        c.hip_stream = stream or None
        c.nin, c.nout, c.nscalars = len(inputs), len(outputs), len(scalars)
        self._call = c
        self._ref = ctypes.byref(c)
        self._run = _lib.ewf_run_call

    @property
    def _stream(self):
        return self._call.hip_stream

    @_stream.setter
    def _stream(self, value) -> None:
        self._call.hip_stream = value.value if isinstance(value, ctypes.c_void_p) else (value or None)

    def launch(self) -> None:
        st = self._run(self._ref)
        if st < 0:
            raise EwfError(st, last_error())


class CallSequence:
    """Prepared calls run in order by one ewf_run_sequence call (the loop runs in the library).
    Keeps the bound calls, and with them their tensors, alive."""

    def __init__(self, calls: Sequence[BoundCall], stream: Optional[int] = None):
        self._calls = list(calls)
        self._arr = (ewf_call * max(1, len(self._calls)))()
        for i, c in enumerate(self._calls):
            ctypes.memmove(ctypes.byref(self._arr[i]), ctypes.byref(c._call), ctypes.sizeof(ewf_call))
            if stream is not None:
                self._arr[i].hip_stream = stream or None
        self._failed = _i32(-1)

    def launch(self) -> None:
        st = _lib.ewf_run_sequence(self._arr, len(self._calls), ctypes.byref(self._failed))
        if st < 0:
            raise EwfError(st, f"call {self._failed.value}: {last_error()}")
