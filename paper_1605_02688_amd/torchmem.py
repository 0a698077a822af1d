"""PyTorch as the owner of device memory for the library's callers here (tests, bench, smoke):
binds a workload's host buffers to device tensors (same bytes, same strided views), allocates
outputs of the shapes the library infers and a workspace of the size a plan asks for.  Argument
plumbing only; every step of the path runs in the library's kernels."""
from __future__ import annotations

import numpy as np
import torch

from . import ewf

_TORCH = {"f32": torch.float32, "f16": torch.float16, "i32": torch.int32}


def device_inputs(w, device="cuda"):
    """(device buffers, one strided view per graph input) of workload `w`."""
    bufs = [torch.from_numpy(np.ascontiguousarray(b)).to(device) for b in w.buffers]
    views = [torch.as_strided(bufs[v.buffer].view(-1), v.shape, v.strides, v.offset) for v in w.views]
    return bufs, views


def alloc_outputs(expr, spec, inputs, device="cuda", fill=None):
    outs = []
    for (_v, storage), shape in zip(spec.outputs, expr.output_shapes(inputs)):
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


def run_workload(w, expr=None, **opts):
    """Runs workload `w` once; returns (expression, outputs on the host as numpy arrays)."""
    expr = expr or ewf.Expression(w.spec, **opts)
    _bufs, ins = device_inputs(w)
    outs = alloc_outputs(expr, w.spec, ins)
    ws = make_workspace(expr, ins, outs)
    expr.run(ins, outs, w.scalars, ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return expr, [o.cpu().numpy() for o in outs]
