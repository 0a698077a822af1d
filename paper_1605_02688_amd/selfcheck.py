"""Build-time check: generate and compile, for gfx950, the kernels of the five benchmark
workloads and of the three backward workloads at their full shapes.  Needs no GPU: planning inspects pointers only for alignment
and aliasing, so synthetic addresses stand in for device memory."""
from __future__ import annotations

from . import ewf


def _contig(shape):
    st, acc = [], 1
    for e in reversed(shape):
        st.append(acc)
        acc *= e
    return tuple(reversed(st))


def plan_layout(expr, spec, views, itemsizes):
    """Plans `expr` for inputs laid out as `views` (buffer id, element offset, shape, strides)
    at made-up, well-aligned addresses.  Returns (workspace bytes, plan info)."""
    base, addr = 0x7F0000000000, {}
    ins = []
    for v, sz in zip(views, itemsizes):
        if v.buffer not in addr:
            addr[v.buffer] = base
            base += 1 << 32
        ins.append(ewf.TensorRef(addr[v.buffer] + v.offset * sz, tuple(v.shape), tuple(v.strides)))
    outs = []
    for shape in expr.output_shapes(ins):
        outs.append(ewf.TensorRef(base, shape, _contig(shape)))
        base += 1 << 32
    ws = expr.plan(ins, outs)
    return ws, expr.info()


def compile_all_workload_kernels(verbose: bool = False) -> int:
    from workloads import configs as wl     # data-only descriptions of the workloads
    count = 0
    for name, make in list(wl.FULL_SIZE.items()) + list(wl.BACKWARD.items()):
        w = wl.layout_only(make)
        expr = ewf.Expression(w.spec)
        ws, info = plan_layout(expr, w.spec, w.views, [w.buffers[v.buffer].itemsize for v in w.views])
        if verbose:
            print(name, "workspace", ws, info)
        count += 1
    return count


if __name__ == "__main__":
    compile_all_workload_kernels(verbose=True)
