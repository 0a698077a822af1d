"""Shared helpers of the GPU parity tests: binds a workload's host buffers to device tensors
(same bytes, same strided views), runs the library through its C ABI binding, runs the
oracle on the host arrays, compares."""
from __future__ import annotations

import numpy as np
import torch

from paper_1605_02688_amd import ewf
from workloads import configs as wl

_TORCH = {"f32": torch.float32, "f16": torch.float16, "i32": torch.int32}


def device_inputs(w, device="cuda"):
    bufs = [torch.from_numpy(np.ascontiguousarray(b)).to(device) for b in w.buffers]
    views = [torch.as_strided(bufs[v.buffer].view(-1), v.shape, v.strides, v.offset) for v in w.views]
    return bufs, views


def alloc_outputs(expr, spec, inputs, device="cuda", fill=None):
    outs = []
    for (v, storage), shape in zip(spec.outputs, expr.output_shapes(inputs)):
        t = torch.empty(shape, dtype=_TORCH[storage], device=device)
        if fill is not None:
            t.fill_(fill)
        outs.append(t)
    return outs


def make_workspace(expr, inputs, outputs, device="cuda"):
    nbytes = expr.plan(inputs, outputs)
    if nbytes == 0:
        return None
    ws = torch.empty((nbytes + 3) // 4, dtype=torch.int32, device=device)
    ewf.workspace_init(ws.data_ptr(), ws.numel() * 4, torch.cuda.current_stream().cuda_stream)
    return ws


def run_gpu(w, expr=None, **opts):
    """Returns (expression, outputs on the host as numpy arrays)."""
    expr = expr or ewf.Expression(w.spec, **opts)
    _bufs, ins = device_inputs(w)
    outs = alloc_outputs(expr, w.spec, ins)
    ws = make_workspace(expr, ins, outs)
    expr.run(ins, outs, w.scalars, ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return expr, [o.cpu().numpy() for o in outs]


def compare(name, got, want, rtol, atol):
    """|got - want| <= atol + rtol*|want| element by element; NaN matches NaN; exact when both
    tolerances are zero.  Returns (max abs error, max rel error)."""
    assert got.shape == want.shape, (name, got.shape, want.shape)
    assert got.dtype == want.dtype, (name, got.dtype, want.dtype)
    if rtol == 0 and atol == 0:
        assert np.array_equal(got, want), f"{name}: integer/exact output differs at {np.argwhere(got != want)[:5]}"
        return 0.0, 0.0
    g = got.astype(np.float64); o = want.astype(np.float64)
    both_nan = np.isnan(g) & np.isnan(o)
    same_inf = np.isinf(o) & (g == o)
    err = np.where(both_nan | same_inf, 0.0, np.abs(g - o))
    lim = atol + rtol * np.abs(np.where(np.isfinite(o), o, 0.0))
    bad = ~(err <= lim)
    if bad.any():
        idx = np.argwhere(bad)[:5]
        raise AssertionError(f"{name}: {int(bad.sum())} of {bad.size} elements out of tolerance "
                             f"(rtol={rtol}, atol={atol}); first at {idx.tolist()}: got {g[bad][:5]}, want {o[bad][:5]}")
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(np.abs(o) > 0, err / np.abs(o), 0.0)
    return float(err.max(initial=0.0)), float(rel.max(initial=0.0))


def check_workload(w, oracle, nthreads=8, **opts):
    expr, got = run_gpu(w, **opts)
    want = oracle.evaluate(w.oracle_spec or w.spec, wl.host_inputs(w), w.scalars, nthreads=nthreads)
    stats = {}
    for name, g, o, (rtol, atol) in zip(w.out_names, got, want, w.tol):
        stats[name] = compare(f"{w.name}.{name}", g, o, rtol, atol)
    return expr, stats
