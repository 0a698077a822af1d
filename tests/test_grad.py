"""Reverse-mode differentiation of the scalar graph (paper section 2.1.3), checked without a
GPU: the library appends the gradient nodes, the node list is read back as a plain
description, the CPU oracle evaluates it, and the result is compared with finite differences
of the oracle's own forward evaluation (the paper's section 2.4 names exactly this check:
symbolic gradients against numeric evaluations) and with hand-derived closed forms."""
import numpy as np
import pytest

from paper_1605_02688_amd import ewf
from workloads import GraphSpec

H = 2.0 ** -6


def grid(rng, shape, lo, hi):
    """float32 values on a 2^-9 grid (so that x +- H and x +- H/2 are exact)."""
    return (np.round(rng.uniform(lo, hi, shape) * 512) / 512).astype(np.float32)


def numeric_grad(oracle, fwd_spec, inputs, cot, k):
    """Richardson-extrapolated central differences of L = sum_j <cot_j, y_j> with respect to
    every element of inputs[k]."""
    def L(xs):
        ys = oracle.evaluate(fwd_spec, xs)
        return sum(float((c.astype(np.float64) * y.astype(np.float64)).sum()) for c, y in zip(cot, ys))
    g = np.zeros(inputs[k].shape)
    for idx in np.ndindex(*inputs[k].shape):
        d = []
        for h in (H, H / 2):
            xp = [a.copy() for a in inputs]; xm = [a.copy() for a in inputs]
            xp[k][idx] += np.float32(h); xm[k][idx] -= np.float32(h)
            d.append((L(xp) - L(xm)) / (2 * h))
        g[idx] = (4 * d[1] - d[0]) / 3
    return g


def check(oracle, build, inputs, wrt, cot_shapes=None, tol=3e-3):
    """build(s, xs) -> list of forward values.  Differentiates with respect to inputs `wrt`."""
    rng = np.random.default_rng(len(inputs) * 7 + len(wrt))
    nd = inputs[0].ndim
    def fresh():
        s = GraphSpec(nd)
        xs = [s.input("f32", tuple(e == 1 and any(a.shape[d] > 1 for a in inputs) for d, e in enumerate(a.shape))) for a in inputs]
        return s, xs
    s, xs = fresh()
    ys = build(s, xs)
    fwd = GraphSpec(nd); fwd.nodes = list(s.nodes); fwd.n_inputs = s.n_inputs
    for y in ys:
        fwd.output(y, "f32")
    y_vals = oracle.evaluate(fwd, inputs)
    cot = [grid(rng, y.shape, -1, 1) for y in y_vals]
    # the gradient graph: cotangents are further inputs
    cs = [s.input("f32", tuple(e == 1 and nd > 0 and any(a.shape[d] > 1 for a in inputs) for d, e in enumerate(c.shape))) for c in cot]
    gs = s.grad(ys, cs, [xs[k] for k in wrt])
    for g_ in gs:
        s.output(g_, "f32")
    plain = ewf.export_spec(s)
    # reduce outputs without keep have a lower rank: feed cotangents in the full rank
    cot_full = []
    for c, cid in zip(cot, cs):
        cot_full.append(c)
    got = oracle.evaluate(plain, list(inputs) + cot_full)
    for j, k in enumerate(wrt):
        want = numeric_grad(oracle, fwd, inputs, cot, k)
        assert got[j].shape == inputs[k].shape, (got[j].shape, inputs[k].shape)
        err = np.abs(got[j] - want).max()
        scale = max(1.0, np.abs(want).max())
        assert err <= tol * scale, (k, err, got[j], want)


UNARY_DOMAINS = {"neg": (-2, 2), "abs": (0.25, 2), "exp": (-2, 2), "log": (0.5, 3), "log1p": (-0.4, 2), "sqrt": (0.5, 3),
                 "tanh": (-2, 2), "sigmoid": (-3, 3), "expm1": (-2, 2), "sqr": (-2, 2), "recip": (0.5, 3)}


@pytest.mark.parametrize("op", sorted(UNARY_DOMAINS))
def test_unary_vjp_against_finite_differences(op, oracle):
    lo, hi = UNARY_DOMAINS[op]
    rng = np.random.default_rng(5)
    x = grid(rng, (3, 4), lo, hi)
    if op == "abs":
        x[0, :] *= -1
    check(oracle, lambda s, xs: [s.apply(op, xs[0])], [x], [0])


@pytest.mark.parametrize("op", ["add", "sub", "mul", "div", "max", "min", "pow"])
def test_binary_vjp_against_finite_differences(op, oracle):
    rng = np.random.default_rng(6)
    a = grid(rng, (3, 4), 0.5, 2.5)
    b = grid(rng, (3, 4), 0.5, 2.5)
    if op in ("max", "min"):
        b = np.where(np.abs(a - b) < 0.1, b + np.float32(0.25), b).astype(np.float32)   # stay clear of the kink
    check(oracle, lambda s, xs: [s.apply(op, xs[0], xs[1])], [a, b], [0, 1])


def test_where_cast_and_comparisons(oracle):
    rng = np.random.default_rng(7)
    a = grid(rng, (2, 5), -2, 2); b = grid(rng, (2, 5), -2, 2)
    a = np.where(np.abs(a) < 0.1, np.float32(0.5), a).astype(np.float32)
    def build(s, xs):
        c = s.apply("gt", xs[0], s.const(0.0))
        w = s.apply("where", c, s.mul(xs[0], xs[1]), s.apply("tanh", xs[1]))
        return [s.add(w, s.cast(s.cast(xs[0], "i32"), "f32"))]        # the integer detour contributes nothing
    check(oracle, build, [a, b], [0, 1])


def test_broadcast_operands_receive_summed_cotangents(oracle):
    rng = np.random.default_rng(8)
    x = grid(rng, (4, 6), -1, 1); row = grid(rng, (1, 6), -1, 1); col = grid(rng, (4, 1), 0.5, 1.5)
    check(oracle, lambda s, xs: [s.apply("tanh", s.add(s.mul(xs[0], xs[2]), xs[1]))], [x, row, col], [0, 1, 2])


def test_reductions_on_the_path(oracle):
    rng = np.random.default_rng(9)
    x = grid(rng, (3, 5), -1, 1)
    x[:, 2] += np.float32(2.0)                                          # a clear row maximum
    def lse(s, xs):
        m = s.reduce("max", xs[0], (1,), keep=True)
        S = s.reduce("sum", s.apply("exp", s.sub(xs[0], m)), (1,), keep=True)
        return [s.add(m, s.apply("log", S))]
    check(oracle, lse, [x], [0])
    check(oracle, lambda s, xs: [s.reduce("sum", s.apply("sqr", xs[0]), (0,), keep=True), s.reduce("min", xs[0], (1,), keep=True)], [x], [0])


def test_product_reduction_gradient_with_and_without_zeros(oracle):
    rng = np.random.default_rng(10)
    x = grid(rng, (4, 5), 0.5, 1.5) * np.where(rng.random((4, 5)) < 0.5, -1, 1).astype(np.float32)
    x[1, 3] = 0.0                                   # one zero in row 1: only that element has a derivative
    x[2, 0] = 0.0; x[2, 4] = 0.0                    # two zeros in row 2: every derivative is zero
    check(oracle, lambda s, xs: [s.reduce("prod", xs[0], (1,), keep=True)], [x], [0])
    check(oracle, lambda s, xs: [s.reduce("prod", xs[0], (0,), keep=True)], [x], [0])
    check(oracle, lambda s, xs: [s.apply("tanh", s.reduce("prod", s.mul(xs[0], xs[0]), (0, 1), keep=True))], [x[:1] + np.float32(2.0)], [0])
    # and the closed form, exactly: row 0 has no zero
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    (g_,) = s.grad([s.reduce("prod", xi, (1,), keep=True)], [s.const(1.0)], [xi])
    s.output(g_, "f32")
    got, = oracle.evaluate(ewf.export_spec(s), [x])
    x64 = x.astype(np.float64)
    want = np.zeros_like(x64)
    for r in range(4):
        for c in range(5):
            want[r, c] = np.prod(np.delete(x64[r], c))
    assert np.allclose(got, want, rtol=1e-5, atol=0)


def test_softmax_cross_entropy_gradient_is_softmax_minus_one_hot(oracle):
    rng = np.random.default_rng(10)
    rows, V = 6, 9
    x = grid(rng, (rows, V), -2, 2)
    t = rng.integers(0, V, (rows, 1)).astype(np.int32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); ti = s.input("i32", (False, True))
    m = s.reduce("max", xi, (1,), keep=True)
    S = s.reduce("sum", s.apply("exp", s.sub(xi, m)), (1,), keep=True)
    picked = s.reduce("sum", s.apply("where", s.apply("eq", s.iota(1), ti), xi, s.const(0.0)), (1,), keep=True)
    loss = s.apply("neg", s.sub(s.sub(picked, m), s.apply("log", S)))
    mean = s.mul(s.reduce("sum", loss, (0,), keep=True), s.const(1.0 / rows))
    (gx,) = s.grad([mean], [s.const(1.0)], [xi])
    s.output(gx, "f32")
    got = oracle.evaluate(ewf.export_spec(s), [x, t])[0]
    p = np.exp(x.astype(np.float64) - x.max(1, keepdims=True)); p /= p.sum(1, keepdims=True)
    onehot = np.zeros((rows, V)); onehot[np.arange(rows), t[:, 0]] = 1
    assert np.abs(got - (p - onehot) / rows).max() < 1e-6


def test_lstm_cell_gradient(oracle):
    rng = np.random.default_rng(11)
    B, Hh = 2, 3
    P = grid(rng, (B, 4 * Hh), -1, 1); bias = grid(rng, (1, 4 * Hh), -1, 1); cprev = grid(rng, (B, Hh), -1, 1)
    # gate slices are separate operands here (the views are a layout matter, not a calculus one)
    zs = [np.ascontiguousarray(P[:, k * Hh:(k + 1) * Hh]) for k in range(4)]
    bs = [np.ascontiguousarray(bias[:, k * Hh:(k + 1) * Hh]) for k in range(4)]
    def cell(s, xs):
        zi, zf, zo, zg = (s.add(xs[k], xs[4 + k]) for k in range(4))
        c = s.add(s.mul(s.apply("sigmoid", zf), xs[8]), s.mul(s.apply("sigmoid", zi), s.apply("tanh", zg)))
        h = s.mul(s.apply("sigmoid", zo), s.apply("tanh", c))
        return [h, c]
    check(oracle, cell, zs + bs + [cprev], list(range(9)))


def _flags(shape, full):
    return tuple(e == 1 and f > 1 for e, f in zip(shape, full))


def check_narrow(oracle, build, inputs, wrt, cot, tol=3e-3):
    """Like `check`, for cotangents that are constant along axes where their value varies: `cot`
    lists, per differentiated value, a float (a literal cotangent) or an array broadcastable to
    the value's shape.  The gradients must come back with the shape of the inputs."""
    full = tuple(max(a.shape[d] for a in inputs) for d in range(inputs[0].ndim))
    s = GraphSpec(len(full))
    xs = [s.input("f32", _flags(a.shape, full)) for a in inputs]
    ys = build(s, xs)
    fwd = GraphSpec(len(full)); fwd.nodes = list(s.nodes); fwd.n_inputs = s.n_inputs
    for y in ys:
        fwd.output(y, "f32")
    y_vals = oracle.evaluate(fwd, inputs)
    cs, extra = [], []
    for c in cot:
        if isinstance(c, float):
            cs.append(s.const(c))
        else:
            cs.append(s.input("f32", _flags(c.shape, full))); extra.append(c)
    gs = s.grad(ys, cs, [xs[k] for k in wrt])
    for g_ in gs:
        s.output(g_, "f32")
    got = oracle.evaluate(ewf.export_spec(s), list(inputs) + extra)
    # (a value that dropped its reduced axes has a lower rank than its cotangent operand)
    cot_full = [c.reshape(y.shape) if not isinstance(c, float) and c.size == y.size else np.broadcast_to(np.float32(c), y.shape)
                for c, y in zip(cot, y_vals)]
    for j, k in enumerate(wrt):
        want = numeric_grad(oracle, fwd, inputs, cot_full, k)
        assert got[j].shape == inputs[k].shape, (k, got[j].shape, inputs[k].shape)
        err = np.abs(got[j] - want).max()
        assert err <= tol * max(1.0, np.abs(want).max()), (k, err, got[j], want)


def test_cotangent_constant_along_an_axis_the_consumer_spans(oracle):
    """The cotangent of a sum is the same for every summed element: an operand that is itself
    constant along the summed axis receives it once per index (extent times), and an operand that
    varies there receives a gradient of its own shape."""
    rng = np.random.default_rng(12)
    x = grid(rng, (3, 4), -1, 1); b = grid(rng, (1, 4), -1, 1); w = grid(rng, (1, 4), 0.5, 1.5)
    col = grid(rng, (3, 1), -1, 1)
    ybar = grid(rng, (1, 4), -1, 1)
    # y = sum_0(x + b): db = 3 ybar, dx = ybar on every row
    def s0(s, xs): return [s.reduce("sum", s.add(xs[0], xs[1]), (0,), keep=True)]
    check(oracle, s0, [x, b], [0, 1])
    check_narrow(oracle, s0, [x, b], [0, 1], [ybar])
    check_narrow(oracle, s0, [x, b], [0, 1], [1.0])
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); bi = s.input("f32", (True, False)); yb = s.input("f32", (True, False))
    gx, gb = s.grad([s.reduce("sum", s.add(xi, bi), (0,), keep=True)], [yb], [xi, bi])
    s.output(gx, "f32"); s.output(gb, "f32")
    dx, db = oracle.evaluate(ewf.export_spec(s), [x, b, ybar])
    assert dx.shape == (3, 4) and np.array_equal(dx, np.broadcast_to(ybar, (3, 4)))
    assert db.shape == (1, 4) and np.array_equal(db, 3 * ybar)
    # sum((x + b) * b): the factor b is constant along the summed axis as well
    check(oracle, lambda s, xs: [s.reduce("sum", s.mul(s.add(xs[0], xs[1]), xs[1]), (0,), keep=True)], [x, b], [0, 1])
    # mean over both axes of x * w + b, with respect to everything
    def mean(s, xs):
        return [s.mul(s.reduce("sum", s.add(s.mul(xs[0], xs[1]), xs[2]), (0, 1), keep=True), s.const(1.0 / 12))]
    check(oracle, mean, [x, w, b], [0, 1, 2])
    check_narrow(oracle, mean, [x, w, b], [0, 1, 2], [1.0])
    # the same through sub, neg and a column operand; reductions without keep
    check(oracle, lambda s, xs: [s.reduce("sum", s.sub(s.apply("neg", xs[1]), s.add(xs[0], xs[2])), (1,), keep=True)],
          [x, b, col], [0, 1, 2])
    check_narrow(oracle, lambda s, xs: [s.reduce("sum", s.add(xs[0], xs[1]), (0,), keep=False)], [x, b], [0, 1], [ybar])
    # a literal cotangent on a full-rank value, with respect to broadcast operands
    full = lambda s, xs: [s.apply("tanh", s.add(s.mul(xs[0], xs[1]), xs[2]))]
    check_narrow(oracle, full, [x, w, col], [0, 1, 2], [1.0])
    check_narrow(oracle, full, [x, w, col], [0, 1, 2], [ybar])
    # element-wise values only, nothing varies along axis 0 in the cotangent or the operand
    check_narrow(oracle, lambda s, xs: [s.add(xs[0], xs[1])], [x, b], [0, 1], [ybar])
    # a chain of two sums: the inner sum's cotangent is constant along both axes
    check_narrow(oracle, lambda s, xs: [s.reduce("sum", s.reduce("sum", s.add(xs[0], xs[1]), (1,), keep=True), (0,), keep=True)],
                 [x, b], [0, 1], [1.0])
    # max-reduction and product reduction downstream of a broadcast operand
    xm = x.copy(); xm[1, :] += np.float32(3.0)
    check(oracle, lambda s, xs: [s.reduce("max", s.add(xs[0], xs[1]), (0,), keep=True)], [xm, b], [0, 1])
    check(oracle, lambda s, xs: [s.reduce("prod", s.add(xs[0], xs[1]), (0,), keep=True)], [x + np.float32(2.0), b], [0, 1])


def test_conventions_and_errors():
    s = GraphSpec(1)
    x = s.input("f32", (False,)); y = s.input("f32", (False,))
    unused = s.apply("exp", y)
    (g_unrelated,) = s.grad([s.apply("tanh", x)], [s.const(1.0)], [y])       # y does not reach tanh(x)
    s.output(g_unrelated, "f32"); s.output(unused, "f32")
    plain = ewf.export_spec(s)
    assert plain.nodes[plain.outputs[0][0]][0] == "apply"                       # y * 0: a zero with y's pattern
    s = GraphSpec(1)
    i = s.input("i32", (False,))
    s.grad([s.cast(i, "f32")], [s.const(1.0)], [i])
    with pytest.raises(ewf.EwfError) as e:
        ewf.export_spec(s)
    assert e.value.status == ewf.ETYPE
