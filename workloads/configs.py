"""The five benchmark workloads as data: a graph description, seeded host buffers, and the
strided views of those buffers that the graph's inputs are bound to.

The tensors are synthetic stand-ins with the shapes of the paper's convnet (section 4.2,
ImageNet-sized NCHW feature maps) and LSTM language-model (section 4.3, Penn Treebank)
workloads; neither data set is needed or used.  Nothing here evaluates an expression.

Seeds: 160502688 + workload number.  Draws come from ``torch.Generator`` on the CPU so that
very large tensors are produced quickly; the arrays returned are numpy.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Sequence, Tuple

import numpy as np
import torch

from .graphspec import GraphSpec

SEED0 = 160502688

# tolerances |got - want| <= atol + rtol * |want| by output class
TOL_F32_ELEMWISE = (2e-6, 1e-6)
TOL_F32_REDUCE = (1e-5, 1e-6)
TOL_F16 = (2e-3, 1e-3)
TOL_EXACT = (0.0, 0.0)


@dataclass
class View:
    """Input k of the graph is ``buffers[buffer]`` seen through (offset, shape, strides),
    all counted in elements."""
    buffer: int
    offset: int
    shape: Tuple[int, ...]
    strides: Tuple[int, ...]


@dataclass
class Workload:
    name: str
    spec: GraphSpec
    buffers: List[np.ndarray]
    views: List[View]
    scalars: List[float]
    out_names: List[str]
    tol: List[Tuple[float, float]]
    elements: int                 # unit of work: output coordinates of the element-wise part
    algorithmic_bytes: int        # every operand read once at its own size + every output once
    notes: Dict[str, object] = field(default_factory=dict)
    # Backward workloads: ``spec`` asks the evaluator's own differentiation for the gradient,
    # which the oracle does not have; it evaluates this hand-derived description instead.
    oracle_spec: object = None


def host_inputs(w: Workload) -> List[np.ndarray]:
    """numpy views of the host buffers, one per graph input."""
    out = []
    for v in w.views:
        base = w.buffers[v.buffer].reshape(-1)
        item = base.itemsize
        out.append(np.lib.stride_tricks.as_strided(
            base[v.offset:], shape=v.shape, strides=tuple(s * item for s in v.strides),
            writeable=False))
    return out


def _contig_strides(shape: Sequence[int]) -> Tuple[int, ...]:
    st, acc = [], 1
    for e in reversed(shape):
        st.append(acc)
        acc *= e
    return tuple(reversed(st))


def _gen(seed: int) -> torch.Generator:
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    return g


class Placeholder:
    """Stands in for a host buffer when only the layout is wanted (``data=False``)."""

    def __init__(self, shape, dtype):
        self.shape = tuple(shape)
        self.dtype = np.dtype(dtype)
        self.itemsize = self.dtype.itemsize
        self.nbytes = int(np.prod(self.shape)) * self.itemsize


_DATA = True


def _uniform(g, shape, lo, hi, dtype=torch.float32):
    if not _DATA:
        return Placeholder(shape, np.float16 if dtype == torch.float16 else np.float32)
    t = torch.rand(tuple(shape), generator=g, dtype=torch.float32) * (hi - lo) + lo
    return t.to(dtype).numpy()


def _normal(g, shape, std=1.0):
    if not _DATA:
        return Placeholder(shape, np.float32)
    return (torch.randn(tuple(shape), generator=g, dtype=torch.float32) * std).numpy()


def layout_only(make, *args, **kw) -> "Workload":
    """Builds a workload description without drawing its tensors."""
    global _DATA
    _DATA = False
    try:
        return make(*args, **kw)
    finally:
        _DATA = True


def _full_view(buf_index: int, shape: Sequence[int]) -> View:
    return View(buf_index, 0, tuple(shape), _contig_strides(shape))


def _nbytes(arrs) -> int:
    return int(sum(a.nbytes for a in arrs))


# --------------------------------------------------------------------------- workload 1

def c1_affine_tanh(rows: int = 1024, cols: int = 256, a: float = 0.5, a_form: str = "scalar") -> Workload:
    """out = tanh(a * X + b); X [rows, cols], b [1, cols] broadcast over dim 0.
    ``a_form``: "scalar" (run-time scalar), "const" (literal) or "tensor" ([1,1] operand)."""
    g = _gen(SEED0 + 1)
    X = _uniform(g, (rows, cols), -1.0, 1.0)
    b = _uniform(g, (1, cols), -1.0, 1.0)
    s = GraphSpec(2)
    x_ = s.input("f32", (False, False))
    b_ = s.input("f32", (True, False))
    buffers, views, scalars = [X, b], [_full_view(0, X.shape), _full_view(1, b.shape)], []
    if a_form == "scalar":
        a_ = s.scalar("f32"); scalars = [a]
    elif a_form == "const":
        a_ = s.const(a, "f32")
    else:
        a_ = s.input("f32", (True, True))
        buffers.append(np.full((1, 1), a, np.float32)); views.append(_full_view(2, (1, 1)))
    out = s.apply("tanh", s.add(s.mul(a_, x_), b_))
    s.output(out, "f32")
    n = rows * cols
    return Workload("c1_affine_tanh", s, buffers, views, scalars, ["out"], [TOL_F32_ELEMWISE],
                    n, X.nbytes + b.nbytes + n * 4)


# --------------------------------------------------------------------------- workload 2

def c2_lstm_cell(batch: int = 64, hidden: int = 1024) -> Workload:
    """LSTM cell point-wise part.  P [batch, 4*hidden] holds the gate pre-activations as
    column blocks in the order i, f, o, g; the four gates are slice views of P (and of the
    bias row), not copies."""
    g = _gen(SEED0 + 2)
    P = _normal(g, (batch, 4 * hidden))
    bias = _normal(g, (1, 4 * hidden))
    c_prev = _normal(g, (batch, hidden))
    s = GraphSpec(2)
    p_ = [s.input("f32", (False, False)) for _ in range(4)]
    b_ = [s.input("f32", (True, False)) for _ in range(4)]
    cp = s.input("f32", (False, False))
    z = [s.add(p_[k], b_[k]) for k in range(4)]
    i_ = s.apply("sigmoid", z[0]); f_ = s.apply("sigmoid", z[1]); o_ = s.apply("sigmoid", z[2])
    g_ = s.apply("tanh", z[3])
    c = s.add(s.mul(f_, cp), s.mul(i_, g_))
    h = s.mul(o_, s.apply("tanh", c))
    s.output(h, "f32"); s.output(c, "f32")
    views = [View(0, k * hidden, (batch, hidden), (4 * hidden, 1)) for k in range(4)]
    views += [View(1, k * hidden, (1, hidden), (4 * hidden, 1)) for k in range(4)]
    views += [_full_view(2, c_prev.shape)]
    n = batch * hidden
    return Workload("c2_lstm_cell", s, [P, bias, c_prev], views, [], ["h", "c"],
                    [TOL_F32_ELEMWISE, TOL_F32_ELEMWISE], n,
                    P.nbytes + bias.nbytes + c_prev.nbytes + 2 * n * 4)


# --------------------------------------------------------------------------- workload 3

def c3_softmax_xent(rows: int = 1280, vocab: int = 10000, std: float = 2.0) -> Workload:
    """Row max, arg-max, exp-sum, log-softmax at the target, per-row loss and mean loss."""
    g = _gen(SEED0 + 3)
    logits = _normal(g, (rows, vocab), std)
    targets = (torch.randint(0, vocab, (rows, 1), generator=g, dtype=torch.int32).numpy()
               if _DATA else Placeholder((rows, 1), np.int32))
    s = GraphSpec(2)
    x = s.input("f32", (False, False))
    t = s.input("i32", (False, True))
    m = s.reduce("max", x, (1,))
    am = s.reduce("argmax", x, (1,))
    sel = s.apply("where", s.apply("eq", s.iota(1), t), x, s.const(0.0))
    xt = s.reduce("sum", sel, (1,))
    S = s.reduce("sum", s.apply("exp", s.sub(x, m)), (1,))
    lsm = s.sub(s.sub(xt, m), s.apply("log", S))
    loss = s.apply("neg", lsm)
    mean = s.div(s.reduce("sum", loss, (0,)), s.const(float(rows)))
    for v in (m, S, lsm, loss, mean):
        s.output(v, "f32")
    s.output(am, "i32")
    nbytes = logits.nbytes + targets.nbytes + 4 * rows * 4 + 4 + rows * 4
    return Workload("c3_softmax_xent", s, [logits, targets],
                    [_full_view(0, logits.shape), _full_view(1, targets.shape)], [],
                    ["rowmax", "expsum", "logsoftmax_at_target", "loss", "mean_loss", "argmax"],
                    [TOL_F32_REDUCE] * 5 + [TOL_EXACT], rows * vocab, nbytes)


# --------------------------------------------------------------------------- workload 4

def c4_bias_relu_chansum(n: int = 128, c: int = 64, h: int = 112, w: int = 112) -> Workload:
    """Y = max(0, X*s + t) on NCHW with per-channel s, t; plus the per-channel sum of Y."""
    g = _gen(SEED0 + 4)
    X = _normal(g, (n, c, h, w))
    sc = _uniform(g, (1, c, 1, 1), 0.5, 1.5)
    sh = _uniform(g, (1, c, 1, 1), -0.5, 0.5)
    s = GraphSpec(4)
    x_ = s.input("f32", (False,) * 4)
    s_ = s.input("f32", (True, False, True, True))
    t_ = s.input("f32", (True, False, True, True))
    y = s.apply("max", s.const(0.0), s.add(s.mul(x_, s_), t_))
    tot = s.reduce("sum", y, (0, 2, 3))
    s.output(y, "f32"); s.output(tot, "f32")
    ne = n * c * h * w
    return Workload("c4_bias_relu_chansum", s, [X, sc, sh],
                    [_full_view(0, X.shape), _full_view(1, sc.shape), _full_view(2, sh.shape)], [],
                    ["Y", "channel_sum"], [TOL_F32_ELEMWISE, TOL_F32_REDUCE], ne,
                    X.nbytes + sc.nbytes + sh.nbytes + ne * 4 + c * 4)


# --------------------------------------------------------------------------- workload 5

def c5_stress(n: int = 64, c: int = 256, h: int = 56, w: int = 56, reading: str = "A",
              bcast: str = "hw") -> Workload:
    """Six inputs, 21 scalar operations, float16 storage.

    x0..x2 contiguous NCHW; x3 a permuted view presented as logical NCHW:
      reading "A": the buffer is contiguous [n, h, w, c] (channels last);
      reading "B": the view is dimshuffle(0,2,3,1) of a contiguous [n, w, c, h] base.
    x4, x5 broadcast: ``bcast="hw"``: x4 [1,c,1,w], x5 [1,c,h,1]; ``bcast="c"``: both [1,c,1,1].
    """
    g = _gen(SEED0 + 5)
    shape = (n, c, h, w)
    xs = [_uniform(g, shape, -2.0, 2.0, torch.float16) for _ in range(3)]
    if reading == "A":
        base3 = _uniform(g, (n, h, w, c), -2.0, 2.0, torch.float16)
        v3 = View(3, 0, shape, (h * w * c, 1, w * c, c))
    elif reading == "contiguous":       # diagnostic only: no permuted operand
        base3 = _uniform(g, shape, -2.0, 2.0, torch.float16)
        v3 = View(3, 0, shape, _contig_strides(shape))
    else:
        base3 = _uniform(g, (n, w, c, h), -2.0, 2.0, torch.float16)
        v3 = View(3, 0, shape, (w * c * h, h, 1, c * h))
    if bcast == "hw":
        s4, s5 = (1, c, 1, w), (1, c, h, 1)
        f4, f5 = (True, False, True, False), (True, False, False, True)
    else:
        s4 = s5 = (1, c, 1, 1)
        f4 = f5 = (True, False, True, True)
    x4 = _uniform(g, s4, -2.0, 2.0, torch.float16)
    x5 = _uniform(g, s5, -2.0, 2.0, torch.float16)
    s = GraphSpec(4)
    i0, i1, i2, i3 = (s.input("f16", (False,) * 4) for _ in range(4))
    i4 = s.input("f16", f4)
    i5 = s.input("f16", f5)
    u = s.add(s.mul(i0, i4), i5)
    sp = s.apply("log1p", s.apply("exp", u))
    q = s.apply("pow", s.add(s.mul(i1, i1), s.const(1.0)), s.mul(s.const(0.5), i2))
    m = s.apply("where", s.apply("gt", i3, s.const(0.0)), sp, q)
    e = s.apply("exp", s.mul(s.mul(s.const(-0.5), i3), i3))
    r = s.add(s.mul(m, e), s.apply("log1p", s.mul(i2, i2)))
    out = s.apply("where", s.apply("gt", i0, i1), r, s.add(s.mul(r, i4), i5))
    s.output(out, "f16")
    ne = n * c * h * w
    buffers = xs + [base3, x4, x5]
    views = [_full_view(k, shape) for k in range(3)] + [v3, _full_view(4, s4), _full_view(5, s5)]
    return Workload(f"c5_stress_{reading}", s, buffers, views, [], ["out"], [TOL_F16], ne,
                    _nbytes(buffers) + ne * 2, {"reading": reading, "bcast": bcast})


# --------------------------------------------------------------------------- backward passes
#
# The paper's benchmarks time forward and backward passes (section 4.2), and its gradients are
# built symbolically (section 2.1.3).  Each workload below gives two descriptions of the same
# backward computation: one that asks the evaluator to differentiate the forward expression,
# and one written out by hand from the chain rule for the oracle.

def c2_lstm_cell_backward(batch: int = 64, hidden: int = 1024) -> Workload:
    """Gradients of the LSTM cell's point-wise part: given dh, dc (cotangents of h and c),
    the cotangents of the four gate pre-activations, of the bias (summed over the batch) and
    of c_prev."""
    g = _gen(SEED0 + 12)
    P = _normal(g, (batch, 4 * hidden))
    bias = _normal(g, (1, 4 * hidden))
    c_prev = _normal(g, (batch, hidden))
    dh = _normal(g, (batch, hidden))
    dc = _normal(g, (batch, hidden))

    def forward(s):
        p_ = [s.input("f32", (False, False)) for _ in range(4)]
        b_ = [s.input("f32", (True, False)) for _ in range(4)]
        cp = s.input("f32", (False, False))
        dh_ = s.input("f32", (False, False)); dc_ = s.input("f32", (False, False))
        z = [s.add(p_[k], b_[k]) for k in range(4)]
        i_ = s.apply("sigmoid", z[0]); f_ = s.apply("sigmoid", z[1]); o_ = s.apply("sigmoid", z[2])
        g_ = s.apply("tanh", z[3])
        c = s.add(s.mul(f_, cp), s.mul(i_, g_))
        tc = s.apply("tanh", c)
        h = s.mul(o_, tc)
        return p_, b_, cp, dh_, dc_, (i_, f_, o_, g_, tc), h, c

    s = GraphSpec(2)
    p_, b_, cp, dh_, dc_, _gates, h, c = forward(s)
    grads = s.grad([h, c], [dh_, dc_], p_ + b_ + [cp])
    for v in grads:
        s.output(v, "f32")

    r = GraphSpec(2)
    p_, b_, cp, dh_, dc_, (i_, f_, o_, g_, tc), h, c = forward(r)
    one = r.const(1.0)
    dct = r.add(dc_, r.mul(r.mul(dh_, o_), r.sub(one, r.mul(tc, tc))))
    dzo = r.mul(r.mul(dh_, tc), r.mul(o_, r.sub(one, o_)))
    dzi = r.mul(r.mul(dct, g_), r.mul(i_, r.sub(one, i_)))
    dzf = r.mul(r.mul(dct, cp), r.mul(f_, r.sub(one, f_)))
    dzg = r.mul(r.mul(dct, i_), r.sub(one, r.mul(g_, g_)))
    dz = [dzi, dzf, dzo, dzg]
    for v in dz:
        r.output(v, "f32")
    for v in dz:
        r.output(r.reduce("sum", v, (0,), keep=True), "f32")
    r.output(r.mul(dct, f_), "f32")

    views = [View(0, k * hidden, (batch, hidden), (4 * hidden, 1)) for k in range(4)]
    views += [View(1, k * hidden, (1, hidden), (4 * hidden, 1)) for k in range(4)]
    views += [_full_view(2, c_prev.shape), _full_view(3, dh.shape), _full_view(4, dc.shape)]
    n = batch * hidden
    names = [f"dz_{k}" for k in "ifog"] + [f"dbias_{k}" for k in "ifog"] + ["dc_prev"]
    tol = [TOL_F32_ELEMWISE] * 4 + [TOL_F32_REDUCE] * 4 + [TOL_F32_ELEMWISE]
    return Workload("c2_lstm_cell_backward", s, [P, bias, c_prev, dh, dc], views, [], names, tol, n,
                    _nbytes([P, bias, c_prev, dh, dc]) + 5 * n * 4 + 4 * hidden * 4, oracle_spec=r)


def c3_softmax_xent_backward(rows: int = 1280, vocab: int = 10000, std: float = 2.0) -> Workload:
    """Gradient of the mean cross-entropy loss with respect to the logits: (softmax - onehot) / rows."""
    g = _gen(SEED0 + 13)
    logits = _normal(g, (rows, vocab), std)
    targets = (torch.randint(0, vocab, (rows, 1), generator=g, dtype=torch.int32).numpy()
               if _DATA else Placeholder((rows, 1), np.int32))
    s = GraphSpec(2)
    x = s.input("f32", (False, False)); t = s.input("i32", (False, True))
    m = s.reduce("max", x, (1,), keep=True)
    S = s.reduce("sum", s.apply("exp", s.sub(x, m)), (1,), keep=True)
    xt = s.reduce("sum", s.apply("where", s.apply("eq", s.iota(1), t), x, s.const(0.0)), (1,), keep=True)
    loss = s.apply("neg", s.sub(s.sub(xt, m), s.apply("log", S)))
    mean = s.div(s.reduce("sum", loss, (0,), keep=True), s.const(float(rows)))
    (dx,) = s.grad([mean], [s.const(1.0)], [x])
    s.output(dx, "f32")

    r = GraphSpec(2)
    x = r.input("f32", (False, False)); t = r.input("i32", (False, True))
    m = r.reduce("max", x, (1,), keep=True)
    e = r.apply("exp", r.sub(x, m))
    p = r.div(e, r.reduce("sum", e, (1,), keep=True))
    onehot = r.apply("where", r.apply("eq", r.iota(1), t), r.const(1.0), r.const(0.0))
    r.output(r.div(r.sub(p, onehot), r.const(float(rows))), "f32")
    return Workload("c3_softmax_xent_backward", s, [logits, targets],
                    [_full_view(0, logits.shape), _full_view(1, targets.shape)], [], ["dlogits"],
                    [(1e-5, 1e-9)], rows * vocab, 2 * logits.nbytes + targets.nbytes, oracle_spec=r)


def c4_bias_relu_chansum_backward(n: int = 128, c: int = 64, h: int = 112, w: int = 112) -> Workload:
    """Gradients of Y = max(0, X*s + t) and its per-channel sum: given dY and the cotangent of
    the channel sums, the cotangent of X and the per-channel cotangents of s and t."""
    g = _gen(SEED0 + 14)
    X = _normal(g, (n, c, h, w))
    sc = _uniform(g, (1, c, 1, 1), 0.5, 1.5)
    sh = _uniform(g, (1, c, 1, 1), -0.5, 0.5)
    dY = _normal(g, (n, c, h, w))
    dsum = _normal(g, (1, c, 1, 1))
    chan = (True, False, True, True)
    s = GraphSpec(4)
    x_ = s.input("f32", (False,) * 4); s_ = s.input("f32", chan); t_ = s.input("f32", chan)
    dy_ = s.input("f32", (False,) * 4); ds_ = s.input("f32", chan)
    y = s.apply("max", s.const(0.0), s.add(s.mul(x_, s_), t_))
    tot = s.reduce("sum", y, (0, 2, 3), keep=True)
    gx, gs, gt = s.grad([y, tot], [dy_, ds_], [x_, s_, t_])
    s.output(gx, "f32"); s.output(gs, "f32"); s.output(gt, "f32")

    r = GraphSpec(4)
    x_ = r.input("f32", (False,) * 4); s_ = r.input("f32", chan); t_ = r.input("f32", chan)
    dy_ = r.input("f32", (False,) * 4); ds_ = r.input("f32", chan)
    z = r.add(r.mul(x_, s_), t_)
    gz = r.apply("where", r.apply("gt", z, r.const(0.0)), r.add(dy_, ds_), r.const(0.0))
    r.output(r.mul(gz, s_), "f32")
    r.output(r.reduce("sum", r.mul(gz, x_), (0, 2, 3), keep=True), "f32")
    r.output(r.reduce("sum", gz, (0, 2, 3), keep=True), "f32")
    ne = n * c * h * w
    bufs = [X, sc, sh, dY, dsum]
    return Workload("c4_bias_relu_chansum_backward", s, bufs, [_full_view(k, b.shape) for k, b in enumerate(bufs)], [],
                    ["dX", "ds", "dt"], [TOL_F32_ELEMWISE, TOL_F32_REDUCE, TOL_F32_REDUCE], ne,
                    _nbytes(bufs) + ne * 4 + 2 * c * 4, oracle_spec=r)


# --------------------------------------------------------------------------- a plan in stages
#
# Batch normalisation of a matrix over its rows (the paper's convnets normalise activations this
# way; section 2.2.1 states what fusion is for: not to loop over a tensor several times).  The
# statistics are reductions over the outer axis and the normalised tensor needs them at every
# element, so no single kernel covers it: the evaluator has to split it into passes.

def batch_norm_axis0(rows: int = 65536, cols: int = 1024, storage: str = "f32") -> Workload:
    """mean and (biased) variance over axis 0 and the normalised tensor, float32 [rows, cols] N(0.5, 2)."""
    g = _gen(SEED0 + 21)
    X = _normal(g, (rows, cols), 2.0)
    if _DATA:
        X = (X + np.float32(0.5)).astype(np.float16 if storage == "f16" else np.float32)
    elif storage == "f16":
        X = Placeholder((rows, cols), np.float16)
    s = GraphSpec(2)
    x = s.input(storage, (False, False))
    inv_n = s.const(1.0 / rows)
    mean = s.mul(s.reduce("sum", x, (0,), keep=True), inv_n)
    cen = s.sub(x, mean)
    var = s.mul(s.reduce("sum", s.mul(cen, cen), (0,), keep=True), inv_n)
    s.output(s.mul(cen, s.apply("recip", s.apply("sqrt", s.add(var, s.const(1e-5))))), storage)
    s.output(mean, "f32"); s.output(var, "f32")
    n = rows * cols
    return Workload(f"batch_norm_axis0_{storage}", s, [X], [_full_view(0, (rows, cols))], [], ["normalised", "mean", "var"],
                    [TOL_F32_REDUCE if storage == "f32" else TOL_F16, TOL_F32_REDUCE, TOL_F32_REDUCE], n,
                    2 * X.nbytes + 2 * cols * 4)


BACKWARD = {"c2b": c2_lstm_cell_backward, "c3b": c3_softmax_xent_backward, "c4b": c4_bias_relu_chansum_backward}

FULL_SIZE = {
    "c1": c1_affine_tanh, "c2": c2_lstm_cell, "c3": c3_softmax_xent,
    "c4": c4_bias_relu_chansum, "c5a": lambda: c5_stress(reading="A"),
    "c5b": lambda: c5_stress(reading="B"),
}
