"""ctypes front end of the CPU oracle (``ewf_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by the tests, by the smoke check and by the benchmark's
CPU-baseline leg.  Nothing in the GPU library or its binding imports this module, and this
module imports nothing from them.

``evaluate(spec, inputs, scalars)`` takes a graph description (any object with ``ndim``,
``nodes`` and ``outputs`` laid out like ``workloads.GraphSpec``), numpy arrays for the inputs
(any strides, float32 / float16 / int32, rank ``ndim``) and returns one freshly allocated
numpy array per output.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ewf_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")

MAXD = 8

_KIND = {"input": 0, "scalar": 1, "const": 2, "iota": 3, "apply": 4, "cast": 5, "reduce": 6}
_VTYPE = {"f32": 0, "i32": 1}
_STORAGE = {"f32": 0, "f16": 1, "i32": 2}
_NP_STORAGE = {np.dtype(np.float32): 0, np.dtype(np.float16): 1, np.dtype(np.int32): 2}
_STORAGE_NP = {"f32": np.float32, "f16": np.float16, "i32": np.int32}
_OPS = {name: i for i, name in enumerate(
    ["add", "sub", "mul", "div", "neg", "abs", "exp", "log", "log1p", "sqrt", "tanh", "sigmoid",
     "max", "min", "pow", "where", "gt", "ge", "lt", "le", "eq", "ne", "expm1", "sqr", "recip"])}
_REDOPS = {"sum": 0, "max": 1, "min": 2, "prod": 3, "argmax": 4}

_ERR = {-1: "invalid graph", -2: "type error", -3: "shape error", -4: "out of memory"}


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__(f"oracle: {_ERR.get(code, 'error')} ({code})")
        self.code = code


class _Node(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("op", ctypes.c_int32), ("nargs", ctypes.c_int32),
                ("args", ctypes.c_int32 * 3), ("index", ctypes.c_int32),
                ("axes", ctypes.c_uint32), ("cval", ctypes.c_double)]


class _Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("storage", ctypes.c_int32), ("bcast", ctypes.c_uint32),
                ("shape", ctypes.c_int64 * MAXD), ("strides", ctypes.c_int64 * MAXD)]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP).  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_eval.restype = ctypes.c_int
        lib.orc_eval.argtypes = [ctypes.c_int, ctypes.POINTER(ctypes.c_int64),
                                 ctypes.POINTER(_Node), ctypes.c_int,
                                 ctypes.POINTER(_Tensor), ctypes.c_int,
                                 ctypes.POINTER(ctypes.c_double), ctypes.c_int,
                                 ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(_Tensor),
                                 ctypes.c_int, ctypes.c_int]
        lib.orc_double_to_half.restype = ctypes.c_uint16
        lib.orc_double_to_half.argtypes = [ctypes.c_double]
        lib.orc_half_to_double.restype = ctypes.c_double
        lib.orc_half_to_double.argtypes = [ctypes.c_uint16]
        _lib = lib
    return _lib


def double_to_half_bits(x: float) -> int:
    return int(_load().orc_double_to_half(float(x)))


def half_bits_to_double(h: int) -> float:
    return float(_load().orc_half_to_double(int(h)))


def _mask(flags: Sequence[bool]) -> int:
    m = 0
    for d, f in enumerate(flags):
        if f:
            m |= 1 << d
    return m


def _analyse_shapes(spec):
    """Per node: (bcast mask, dropped mask).  A dimension is dropped from an output's shape
    when the value is broadcastable there and a reduce with keep=False removed it."""
    ndim = spec.ndim
    allm = (1 << ndim) - 1
    bc, dr = [], []
    for node in spec.nodes:
        kind = node[0]
        if kind == "input":
            bc.append(_mask(node[3])); dr.append(0)
        elif kind in ("scalar", "const"):
            bc.append(allm); dr.append(0)
        elif kind == "iota":
            bc.append(allm & ~(1 << node[1])); dr.append(0)
        elif kind == "cast":
            bc.append(bc[node[1]]); dr.append(dr[node[1]])
        elif kind == "apply":
            b, u = allm, 0
            for a in node[2]:
                b &= bc[a]; u |= dr[a]
            bc.append(b); dr.append(u & b)
        elif kind == "reduce":
            _, _, arg, axes, keep = node
            am = _mask([d in axes for d in range(ndim)])
            b = bc[arg] | am
            u = dr[arg] | (0 if keep else am)
            bc.append(b); dr.append(u & b)
        else:
            raise ValueError(kind)
    return bc, dr


def evaluate(spec, inputs: Sequence[np.ndarray], scalars: Sequence[float] = (),
             nthreads: int = 1) -> List[np.ndarray]:
    lib = _load()
    ndim = spec.ndim
    if ndim > MAXD:
        raise ValueError("rank too large")
    inputs = [np.asarray(a) for a in inputs]

    # iteration space: what every non-broadcastable dimension measures
    in_nodes = [n for n in spec.nodes if n[0] == "input"]
    if len(in_nodes) != len(inputs):
        raise ValueError("wrong number of inputs")
    full = [1] * ndim
    for node, arr in zip(in_nodes, inputs):
        if arr.ndim != ndim:
            raise OracleError(-3)
        for d in range(ndim):
            if not node[3][d]:
                full[d] = arr.shape[d]

    nodes = (_Node * len(spec.nodes))()
    for i, node in enumerate(spec.nodes):
        n = nodes[i]
        n.kind = _KIND[node[0]]
        if node[0] == "input":
            n.index = node[1]
        elif node[0] == "scalar":
            n.index = node[1]; n.op = _VTYPE[node[2]]
        elif node[0] == "const":
            n.op = _VTYPE[node[1]]; n.cval = node[2]
        elif node[0] == "iota":
            n.index = node[1]
        elif node[0] == "apply":
            n.op = _OPS[node[1]]; n.nargs = len(node[2])
            for k, a in enumerate(node[2]):
                n.args[k] = a
        elif node[0] == "cast":
            n.op = _STORAGE[node[2]]; n.nargs = 1; n.args[0] = node[1]
        elif node[0] == "reduce":
            n.op = _REDOPS[node[1]]; n.nargs = 1; n.args[0] = node[2]
            n.axes = _mask([d in node[3] for d in range(ndim)])

    tin = (_Tensor * max(1, len(inputs)))()
    for k, (node, arr) in enumerate(zip(in_nodes, inputs)):
        if arr.dtype not in _NP_STORAGE or _NP_STORAGE[arr.dtype] != _STORAGE[node[2]]:
            raise OracleError(-2)
        t = tin[k]
        t.data = arr.ctypes.data
        t.storage = _NP_STORAGE[arr.dtype]
        t.bcast = _mask(node[3])
        for d in range(ndim):
            t.shape[d] = arr.shape[d]
            if arr.strides[d] % arr.itemsize:
                raise ValueError("stride is not a whole number of elements")
            t.strides[d] = arr.strides[d] // arr.itemsize

    bc, dr = _analyse_shapes(spec)
    outs_full, tout = [], (_Tensor * max(1, len(spec.outputs)))()
    out_nodes = (ctypes.c_int32 * max(1, len(spec.outputs)))()
    for k, (v, storage) in enumerate(spec.outputs):
        shape = [1 if (bc[v] >> d) & 1 else full[d] for d in range(ndim)]
        arr = np.empty(shape, dtype=_STORAGE_NP[storage])
        outs_full.append(arr)
        out_nodes[k] = v
        t = tout[k]
        t.data = arr.ctypes.data
        t.storage = _STORAGE[storage]
        for d in range(ndim):
            t.shape[d] = shape[d]
            t.strides[d] = arr.strides[d] // arr.itemsize

    sc = (ctypes.c_double * max(1, len(scalars)))(*[float(s) for s in scalars])
    fullc = (ctypes.c_int64 * MAXD)(*full)
    rc = lib.orc_eval(ndim, fullc, nodes, len(spec.nodes), tin, len(inputs), sc, len(scalars),
                      out_nodes, tout, len(spec.outputs), int(nthreads))
    if rc != 0:
        raise OracleError(rc)

    results = []
    for (v, _), arr in zip(spec.outputs, outs_full):
        keep_dims = [d for d in range(ndim) if not (dr[v] >> d) & 1]
        results.append(arr.reshape([arr.shape[d] for d in keep_dims]))
    return results
