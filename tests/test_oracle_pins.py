"""Pins for the CPU oracle: closed forms, hand-computed tensors, identities, broadcast and
stride invariants, and brute force against independent numpy float64 expressions.  None of
these tests touches the GPU library."""
import json
import math
import os

import numpy as np
import pytest

from workloads import GraphSpec
from workloads import configs as wl

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")))


def ev1(oracle, spec, inputs, scalars=()):
    return oracle.evaluate(spec, inputs, scalars)


def unary_spec(op, storage="f32", out="f32"):
    s = GraphSpec(1)
    s.output(s.apply(op, s.input(storage, (False,))), out)
    return s


def binary_spec(op, out="f32", storage="f32"):
    s = GraphSpec(1)
    a = s.input(storage, (False,)); b = s.input(storage, (False,))
    s.output(s.apply(op, a, b), out)
    return s


# ------------------------------------------------------------------ closed forms

def test_sigmoid_tanh_closed_forms(oracle):
    xs = np.array([0.0, 1.0, -1.0, 2.0], np.float32)
    got = oracle.evaluate(unary_spec("sigmoid"), [xs])[0]
    want = np.array([GOLD["sigmoid"][str(float(x))] for x in xs])
    assert np.array_equal(got, want.astype(np.float32))
    assert got[0] == 0.5
    xs = np.array([0.5, 1.5, 2.0], np.float32)
    got = oracle.evaluate(unary_spec("tanh"), [xs])[0]
    want = np.array([GOLD["tanh"][str(float(x))] for x in xs])
    assert np.array_equal(got, want.astype(np.float32))


def test_tanh_odd_sigmoid_mirror(oracle):
    x = np.linspace(-9, 9, 181).astype(np.float32)
    t = oracle.evaluate(unary_spec("tanh"), [x])[0]
    assert np.array_equal(t, -t[::-1])
    s = oracle.evaluate(unary_spec("sigmoid"), [x])[0].astype(np.float64)
    assert np.allclose(s + s[::-1], 1.0, rtol=0, atol=1e-7)
    # saturation without overflow
    big = np.array([-200.0, 200.0], np.float32)
    assert np.array_equal(oracle.evaluate(unary_spec("sigmoid"), [big])[0], [0.0, 1.0])


def test_c1_tiny_hand_computed(oracle):
    w = wl.c1_affine_tanh(rows=2, cols=2)
    X = np.array([[0, 1], [-1, 2]], np.float32)
    b = np.array([[0, 1]], np.float32)
    got = oracle.evaluate(w.spec, [X, b], [0.5])[0]
    assert np.array_equal(got, np.array(GOLD["c1_tiny"]).astype(np.float32))


@pytest.mark.parametrize("key,z,cp", [("zeros_cprev1", (0, 0, 0, 0), 1.0),
                                       ("i1_f-1_o2_g0.5_cprev0.25", (1, -1, 2, 0.5), 0.25)])
def test_c2_tiny_hand_computed(oracle, key, z, cp):
    w = wl.c2_lstm_cell(batch=1, hidden=1)
    P = np.array([z], np.float32)                       # [1, 4]: i, f, o, g
    ins = [P[:, k:k + 1] for k in range(4)] + [np.zeros((1, 1), np.float32)] * 4 + \
          [np.array([[cp]], np.float32)]
    h, c = oracle.evaluate(w.spec, ins)
    cw, hw = GOLD["c2_tiny"][key]
    assert c[0, 0] == np.float32(cw) and h[0, 0] == np.float32(hw)


def test_c2_bias_is_added(oracle):
    # moving the pre-activation into the bias row must not change the result
    w = wl.c2_lstm_cell(batch=1, hidden=1)
    z = (1, -1, 2, 0.5)
    zero = np.zeros((1, 1), np.float32)
    ins = [zero] * 4 + [np.array([[v]], np.float32) for v in z] + [np.array([[0.25]], np.float32)]
    h, c = oracle.evaluate(w.spec, ins)
    cw, hw = GOLD["c2_tiny"]["i1_f-1_o2_g0.5_cprev0.25"]
    assert c[0, 0] == np.float32(cw) and h[0, 0] == np.float32(hw)


def test_c3_tiny_hand_computed(oracle):
    w = wl.c3_softmax_xent(rows=2, vocab=3)
    x = np.array([[1, 2, 3], [1, 2, 3]], np.float32)
    t = np.array([[2], [0]], np.int32)
    m, S, lsm, loss, mean, am = oracle.evaluate(w.spec, [x, t])
    G = GOLD["c3_tiny"]
    assert m.shape == (2,) and mean.shape == () and am.dtype == np.int32
    assert np.array_equal(m, [3, 3]) and np.array_equal(am, [2, 2])
    assert np.array_equal(S, np.float32([G["S"]] * 2))
    assert lsm[0] == np.float32(G["lsm_t2"])
    assert np.array_equal(loss, np.float32([G["loss_t2"], G["loss_t0"]]))
    assert mean == np.float32((G["loss_t2"] + G["loss_t0"]) / 2)


# ------------------------------------------------------------------ identities

def test_softmax_identities(oracle):
    rows, V = 7, 33
    w = wl.c3_softmax_xent(rows=rows, vocab=V)
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((rows, V)) * 2).astype(np.float32)
    t = rng.integers(0, V, (rows, 1)).astype(np.int32)
    m, S, lsm, loss, mean, am = oracle.evaluate(w.spec, [x, t])
    # library special case: log-sum-exp by numpy in float64
    xd = x.astype(np.float64)
    lse = np.log(np.exp(xd - xd.max(1, keepdims=True)).sum(1)) + xd.max(1)
    assert np.allclose(m.astype(np.float64) + np.log(S.astype(np.float64)), lse, rtol=1e-6)
    assert np.array_equal(am, xd.argmax(1))
    assert np.allclose(loss, lse - xd[np.arange(rows), t[:, 0]], rtol=1e-6, atol=1e-7)
    assert (loss >= 0).all()
    # shift invariance: LSE(x + c) = LSE(x) + c, loss unchanged (c exactly representable)
    m2, S2, lsm2, loss2, mean2, am2 = oracle.evaluate(w.spec, [x + np.float32(4.0), t])
    assert np.allclose(loss2, loss, rtol=1e-6, atol=1e-6) and np.array_equal(am2, am)
    assert np.allclose(m2, m + 4.0)
    # softmax rows sum to one: p = exp(x - m) / S summed over the row
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    mm = s.reduce("max", xi, (1,))
    e = s.apply("exp", s.sub(xi, mm))
    p = s.div(e, s.reduce("sum", e, (1,)))
    s.output(s.reduce("sum", p, (1,)), "f32")
    s.output(p, "f32")
    tot, pm = oracle.evaluate(s, [x])
    assert np.allclose(tot, 1.0, rtol=0, atol=1e-7)
    assert pm.shape == (rows, V) and np.allclose(pm.sum(1), 1.0, atol=1e-5)


def test_constant_row_loss_is_log_vocab(oracle):
    V = 10000
    w = wl.c3_softmax_xent(rows=2, vocab=V)
    x = np.full((2, V), 1.25, np.float32)
    t = np.array([[17], [9999]], np.int32)
    m, S, lsm, loss, mean, am = oracle.evaluate(w.spec, [x, t])
    assert np.array_equal(am, [0, 0])                       # ties: first index wins
    assert np.array_equal(S, [V, V])
    assert np.allclose(loss, GOLD["ln_10000"], rtol=1e-7)
    # one dominant logit at the target: loss -> 0
    x[0, 17] = 60.0
    loss = oracle.evaluate(w.spec, [x, t])[3]
    assert 0 <= loss[0] < 1e-20 and oracle.evaluate(w.spec, [x, t])[5][0] == 17


def test_argmax_ties_and_position(oracle):
    s = GraphSpec(2)
    x = s.input("f32", (False, False))
    s.output(s.reduce("argmax", x, (0,)), "i32")
    s.output(s.reduce("argmax", x, (1,), keep=True), "i32")
    a = np.array([[1, 5, 5], [7, 5, 2], [7, 1, 5]], np.float32)
    a0, a1 = oracle.evaluate(s, [a])
    assert np.array_equal(a0, [1, 0, 0]) and a0.shape == (3,)
    assert np.array_equal(a1, [[1], [0], [0]])


def test_out_of_range_target_contributes_zero(oracle):
    w = wl.c3_softmax_xent(rows=1, vocab=3)
    x = np.array([[1, 2, 3]], np.float32)
    lsm = oracle.evaluate(w.spec, [x, np.array([[7]], np.int32)])[2]
    G = GOLD["c3_tiny"]
    assert lsm[0] == np.float32(-G["m"] - math.log(G["S"]))


# ------------------------------------------------------------------ c4 pins

def test_c4_identities(oracle):
    w = wl.c4_bias_relu_chansum(n=3, c=4, h=5, w=6)
    rng = np.random.default_rng(4)
    X = np.abs(rng.integers(-50, 50, (3, 4, 5, 6))).astype(np.float32)
    one = np.ones((1, 4, 1, 1), np.float32); zero = np.zeros((1, 4, 1, 1), np.float32)
    Y, tot = oracle.evaluate(w.spec, [X, one, zero])
    assert np.array_equal(Y, X) and tot.shape == (4,)
    assert np.array_equal(tot, X.sum(axis=(0, 2, 3)))             # integer-valued: exact
    Xs = rng.standard_normal((3, 4, 5, 6)).astype(np.float32)
    sc = rng.uniform(0.5, 1.5, (1, 4, 1, 1)).astype(np.float32)
    sh = rng.uniform(-0.5, 0.5, (1, 4, 1, 1)).astype(np.float32)
    Y, tot = oracle.evaluate(w.spec, [Xs, sc, sh])
    assert (Y >= 0).all()
    ref = np.maximum(0.0, Xs.astype(np.float64) * sc + sh)
    assert np.array_equal(Y, ref.astype(np.float32))
    assert np.allclose(tot, ref.sum(axis=(0, 2, 3)), rtol=1e-7)


def test_c4_statistics_of_generator(oracle):
    # mean of max(0, s z + t), z ~ N(0,1), equals t Phi(t/s) + s phi(t/s)
    w = wl.c4_bias_relu_chansum(n=16, c=3, h=100, w=100)
    X = wl.host_inputs(w)[0]
    for key, (sv, tv) in {"s1_t0": (1, 0), "s1.5_t0.5": (1.5, .5), "s0.5_t-0.5": (.5, -.5)}.items():
        sc = np.full((1, 3, 1, 1), sv, np.float32); sh = np.full((1, 3, 1, 1), tv, np.float32)
        tot = oracle.evaluate(w.spec, [X, sc, sh], nthreads=4)[1]
        assert np.allclose(tot / (16 * 100 * 100), GOLD["relu_mean"][key], rtol=2e-2)


# ------------------------------------------------------------------ broadcast / stride rules

def test_broadcast_equals_tiled(oracle):
    rng = np.random.default_rng(5)
    X = rng.standard_normal((4, 3, 5)).astype(np.float32)
    b = rng.standard_normal((1, 3, 1)).astype(np.float32)
    s = GraphSpec(3)
    s.output(s.apply("tanh", s.mul(s.input("f32", (False,) * 3), s.input("f32", (True, False, True)))), "f32")
    s2 = GraphSpec(3)
    s2.output(s2.apply("tanh", s2.mul(s2.input("f32", (False,) * 3), s2.input("f32", (False,) * 3))), "f32")
    a = oracle.evaluate(s, [X, b])[0]
    bt = np.ascontiguousarray(np.broadcast_to(b, X.shape))
    assert np.array_equal(a, oracle.evaluate(s2, [X, bt])[0])


def test_strided_view_equals_copy_and_transpose(oracle):
    rng = np.random.default_rng(6)
    base = rng.standard_normal((6, 10)).astype(np.float32)
    view = base[1:5, ::3]                                   # sliced, non-contiguous
    s = unary_spec("exp"); s.ndim = 2
    s = GraphSpec(2); s.output(s.apply("exp", s.input("f32", (False, False))), "f32")
    assert np.array_equal(oracle.evaluate(s, [view])[0], oracle.evaluate(s, [view.copy()])[0])
    # f(X^T)^T == f(X)
    assert np.array_equal(oracle.evaluate(s, [base.T])[0].T, oracle.evaluate(s, [base])[0])
    # the transposed view addresses element (i,j) at base[j,i]
    s3 = GraphSpec(2)
    s3.output(s3.sub(s3.input("f32", (False, False)), s3.input("f32", (False, False))), "f32")
    sq = rng.standard_normal((5, 5)).astype(np.float32)
    d = oracle.evaluate(s3, [sq, sq.T])[0]
    assert np.array_equal(d, sq - sq.T) and np.array_equal(d, -d.T)


def test_bcast_flag_is_a_guarantee(oracle):
    s = GraphSpec(2)
    s.output(s.add(s.input("f32", (False, False)), s.input("f32", (False, False))), "f32")
    with pytest.raises(oracle.OracleError) as e:
        oracle.evaluate(s, [np.zeros((3, 4), np.float32), np.zeros((1, 4), np.float32)])
    assert e.value.code == -3
    s = GraphSpec(2)
    s.output(s.add(s.input("f32", (False, False)), s.input("f32", (True, False))), "f32")
    with pytest.raises(oracle.OracleError):
        oracle.evaluate(s, [np.zeros((3, 4), np.float32), np.zeros((3, 4), np.float32)])


def test_c1_forms_of_a_agree(oracle):
    outs = []
    for form in ("scalar", "const", "tensor"):
        w = wl.c1_affine_tanh(rows=9, cols=7, a_form=form)
        outs.append(oracle.evaluate(w.spec, wl.host_inputs(w), w.scalars)[0])
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_c2_views_are_slices_of_P(oracle):
    w = wl.c2_lstm_cell(batch=3, hidden=5)
    ins = wl.host_inputs(w)
    P, bias, cp = w.buffers
    for k in range(4):
        assert np.array_equal(ins[k], P[:, 5 * k:5 * (k + 1)])
        assert np.array_equal(ins[4 + k], bias[:, 5 * k:5 * (k + 1)])
    h, c = oracle.evaluate(w.spec, ins)
    Pd = (P + bias).astype(np.float64) if False else P.astype(np.float64) + bias.astype(np.float64)
    sg = lambda v: 1 / (1 + np.exp(-v))
    i, f, o, g = (Pd[:, 5 * k:5 * (k + 1)] for k in range(4))
    cr = sg(f) * cp + sg(i) * np.tanh(g)
    hr = sg(o) * np.tanh(cr)
    assert np.allclose(c, cr, rtol=1e-6, atol=1e-7) and np.allclose(h, hr, rtol=1e-6, atol=1e-7)


def test_c5_views_and_expression(oracle):
    for reading in ("A", "B"):
        for bc in ("hw", "c"):
            w = wl.c5_stress(n=2, c=4, h=3, w=5, reading=reading, bcast=bc)
            ins = wl.host_inputs(w)
            base3 = w.buffers[3]
            if reading == "A":
                assert np.array_equal(ins[3], base3.transpose(0, 3, 1, 2))
            else:                       # dimshuffle(0,2,3,1) of the [n,w,c,h] base
                assert np.array_equal(ins[3], base3.transpose(0, 2, 3, 1))
            x0, x1, x2, x3, x4, x5 = (a.astype(np.float64) for a in ins)
            u = x0 * x4 + x5
            sp = np.log1p(np.exp(u))
            q = np.power(x1 * x1 + 1, 0.5 * x2)
            m = np.where(x3 > 0, sp, q)
            e = np.exp(-0.5 * x3 * x3)
            r = m * e + np.log1p(x2 * x2)
            ref = np.where(x0 > x1, r, r * x4 + x5)
            got = oracle.evaluate(w.spec, ins)[0]
            assert got.dtype == np.float16
            assert np.array_equal(got, ref.astype(np.float16))


# ------------------------------------------------------------------ reductions

def test_integer_valued_sums_are_exact_any_axes(oracle):
    rng = np.random.default_rng(7)
    X = rng.integers(-100, 100, (5, 6, 7)).astype(np.float32)
    for axes in [(0,), (1,), (2,), (0, 1), (0, 2), (1, 2), (0, 1, 2)]:
        for keep in (False, True):
            s = GraphSpec(3)
            s.output(s.reduce("sum", s.input("f32", (False,) * 3), axes, keep=keep), "f32")
            got = oracle.evaluate(s, [X])[0]
            want = X.astype(np.float64).sum(axis=axes, keepdims=keep)
            assert got.shape == want.shape and np.array_equal(got, want)


def test_reduce_ops_vs_numpy(oracle):
    rng = np.random.default_rng(8)
    X = rng.standard_normal((4, 9)).astype(np.float32)
    for red, fn in (("max", np.max), ("min", np.min), ("prod", np.prod), ("sum", np.sum)):
        for ax in (0, 1):
            s = GraphSpec(2)
            s.output(s.reduce(red, s.input("f32", (False, False)), (ax,)), "f32")
            got = oracle.evaluate(s, [X])[0]
            assert np.allclose(got, fn(X.astype(np.float64), axis=ax), rtol=1e-7)
    # reduce over an axis on which the argument is broadcastable runs over extent 1
    s = GraphSpec(2)
    r = s.reduce("sum", s.input("f32", (False, False)), (1,))
    s.output(s.reduce("sum", r, (0, 1)), "f32")
    assert np.allclose(oracle.evaluate(s, [X])[0], X.astype(np.float64).sum(), rtol=1e-7)
    # reduce of an operand with a strided view (transpose) sums the right elements
    s = GraphSpec(2)
    s.output(s.reduce("sum", s.input("f32", (False, False)), (1,)), "f32")
    assert np.allclose(oracle.evaluate(s, [X.T])[0], X.astype(np.float64).sum(0), rtol=1e-7)


def test_empty_reductions(oracle):
    s = GraphSpec(2)
    s.output(s.reduce("sum", s.input("f32", (False, False)), (1,)), "f32")
    assert np.array_equal(oracle.evaluate(s, [np.zeros((3, 0), np.float32)])[0], [0, 0, 0])
    s = GraphSpec(2)
    s.output(s.reduce("max", s.input("f32", (False, False)), (1,)), "f32")
    with pytest.raises(oracle.OracleError):
        oracle.evaluate(s, [np.zeros((3, 0), np.float32)])


def test_nan_conventions(oracle):
    nan = np.float32("nan")
    a = np.array([1, nan, 3, nan], np.float32); b = np.array([2, 2, nan, nan], np.float32)
    assert np.array_equal(oracle.evaluate(binary_spec("max"), [a, b])[0], np.maximum(a, b), equal_nan=True)
    assert np.array_equal(oracle.evaluate(binary_spec("min"), [a, b])[0], np.minimum(a, b), equal_nan=True)
    s = GraphSpec(1)
    c = s.input("f32", (False,))
    s.output(s.apply("where", c, s.input("f32", (False,)), s.input("f32", (False,))), "f32")
    cond = np.array([0, 1, nan, -0.0], np.float32)
    x = np.array([10, 11, 12, 13], np.float32); y = np.array([nan, nan, 22, 23], np.float32)
    assert np.array_equal(oracle.evaluate(s, [cond, x, y])[0], np.float32([nan, 11, 12, 23]), equal_nan=True)


# ------------------------------------------------------------------ every op, brute force

_UN = {"neg": np.negative, "abs": np.abs, "exp": np.exp, "log": np.log, "log1p": np.log1p,
       "sqrt": np.sqrt, "tanh": np.tanh, "expm1": np.expm1, "sqr": np.square,
       "recip": lambda v: 1.0 / v, "sigmoid": lambda v: 1.0 / (1.0 + np.exp(-v))}
_BIN = {"add": np.add, "sub": np.subtract, "mul": np.multiply, "div": np.divide,
        "max": np.maximum, "min": np.minimum, "pow": np.power}
_CMP = {"gt": np.greater, "ge": np.greater_equal, "lt": np.less, "le": np.less_equal,
        "eq": np.equal, "ne": np.not_equal}


@pytest.mark.parametrize("op", sorted(_UN))
def test_unary_vs_numpy_float64(oracle, op):
    rng = np.random.default_rng(11)
    x = rng.uniform(0.05, 4.0, 257).astype(np.float32)
    if op not in ("log", "sqrt", "recip"):
        x = x * rng.choice([-1, 1], x.shape).astype(np.float32)
    if op == "log1p":
        x = np.where(x < 0, x * np.float32(0.2), x).astype(np.float32)      # stay above -1
    got = oracle.evaluate(unary_spec(op), [x])[0]
    assert np.array_equal(got, _UN[op](x.astype(np.float64)).astype(np.float32))


def test_log1p_small_argument(oracle):
    x = np.float32([1e-7, -1e-7, 3e-10])
    got = oracle.evaluate(unary_spec("log1p"), [x])[0]
    assert np.allclose(got, x.astype(np.float64), rtol=1e-6)       # log(1+x) in f32 would give 0
    assert (got != 0).all()


@pytest.mark.parametrize("op", sorted(_BIN))
def test_binary_vs_numpy_float64(oracle, op):
    rng = np.random.default_rng(12)
    a = rng.uniform(-3, 3, 300).astype(np.float32)
    b = rng.uniform(-3, 3, 300).astype(np.float32)
    if op == "pow":
        a = np.abs(a) + np.float32(0.1)
    got = oracle.evaluate(binary_spec(op), [a, b])[0]
    assert np.array_equal(got, _BIN[op](a.astype(np.float64), b.astype(np.float64)).astype(np.float32))
    if op == "sub":                     # operand order
        assert got[0] == np.float32(np.float64(a[0]) - np.float64(b[0]))


@pytest.mark.parametrize("op", sorted(_CMP))
def test_compare_and_where(oracle, op):
    rng = np.random.default_rng(13)
    a = rng.integers(-3, 3, 200).astype(np.float32)
    b = rng.integers(-3, 3, 200).astype(np.float32)
    got = oracle.evaluate(binary_spec(op, out="i32"), [a, b])[0]
    assert got.dtype == np.int32 and np.array_equal(got, _CMP[op](a, b).astype(np.int32))
    s = GraphSpec(1)
    x = s.input("f32", (False,)); y = s.input("f32", (False,))
    s.output(s.apply("where", s.apply(op, x, y), x, y), "f32")
    assert np.array_equal(oracle.evaluate(s, [a, b])[0], np.where(_CMP[op](a, b), a, b))


def test_int32_arithmetic_and_iota(oracle):
    a = np.array([2**31 - 1, -5, 7, 46341], np.int32); b = np.array([1, 3, -2, 46341], np.int32)
    for op, fn in (("add", np.add), ("sub", np.subtract), ("mul", np.multiply),
                   ("max", np.maximum), ("min", np.minimum)):
        got = oracle.evaluate(binary_spec(op, out="i32", storage="i32"), [a, b])[0]
        with np.errstate(over="ignore"):
            assert np.array_equal(got, fn(a, b)), op            # wraps like two's complement
    s = GraphSpec(3)
    x = s.input("i32", (False, False, False))
    s.output(s.add(s.mul(s.iota(0), s.const(100, "i32")), s.add(s.mul(s.iota(1), s.const(10, "i32")), s.iota(2))), "i32")
    s.output(x, "i32")
    z = np.zeros((2, 3, 4), np.int32)
    io = oracle.evaluate(s, [z])[0]
    i, j, k = np.meshgrid(np.arange(2), np.arange(3), np.arange(4), indexing="ij")
    assert np.array_equal(io, 100 * i + 10 * j + k)


def test_casts(oracle):
    x = np.float32([1.7, -1.7, 0.5, -0.5, 3e9, -3e9, 65520.0, 1e-8, 1.00048828125])
    s = GraphSpec(1); s.output(s.cast(s.input("f32", (False,)), "i32"), "i32")
    assert np.array_equal(oracle.evaluate(s, [x])[0][:6], [1, -1, 0, 0, 2**31 - 1, -2**31])
    s = GraphSpec(1); s.output(s.cast(s.input("f32", (False,)), "f16"), "f32")
    with np.errstate(over="ignore"):
        assert np.array_equal(oracle.evaluate(s, [x])[0], x.astype(np.float16).astype(np.float32))
    i = np.array([16777217, -16777219, 5], np.int32)
    s = GraphSpec(1); s.output(s.cast(s.input("i32", (False,)), "f32"), "f32")
    assert np.array_equal(oracle.evaluate(s, [i])[0], i.astype(np.float32))
    # storage type must match the value type unless a cast says otherwise
    s = GraphSpec(1); s.output(s.input("i32", (False,)), "f32")
    with pytest.raises(oracle.OracleError):
        oracle.evaluate(s, [i])
    s = GraphSpec(1); s.output(s.add(s.input("i32", (False,)), s.input("f32", (False,))), "f32")
    with pytest.raises(oracle.OracleError):
        oracle.evaluate(s, [i, x[:3]])


def test_half_conversions_all_bit_patterns(oracle):
    # every binary16 value widens exactly; numpy's conversion is the independent reference
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float64)
    got = np.array([oracle.half_bits_to_double(int(b)) for b in bits[::7]])
    assert np.array_equal(got, ref[::7], equal_nan=True)
    rng = np.random.default_rng(14)
    xs = np.concatenate([rng.uniform(-70000, 70000, 3000), rng.uniform(-1e-4, 1e-4, 3000),
                         rng.uniform(-7e-8, 7e-8, 500),
                         # exact ties between neighbouring float16 values
                         (ref[1024:3000:13] + ref[1025:3001:13]) / 2, [65504.0, 65519.99, 65520.0, 0.0, -0.0]])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half_bits(float(v)) for v in xs], np.uint16)
    assert np.array_equal(got, want)


def test_f16_storage_round_trip(oracle):
    rng = np.random.default_rng(15)
    a = rng.uniform(-2, 2, 500).astype(np.float16); b = rng.uniform(-2, 2, 500).astype(np.float16)
    got = oracle.evaluate(binary_spec("mul", out="f16", storage="f16"), [a, b])[0]
    assert got.dtype == np.float16
    assert np.array_equal(got, (a.astype(np.float64) * b.astype(np.float64)).astype(np.float16))


# ------------------------------------------------------------------ random graphs, brute force

def _np_eval(spec, inputs, scalars, full):
    """Independent evaluator: numpy float64 broadcasting, keepdims reductions."""
    vals = []
    for node in spec.nodes:
        k = node[0]
        if k == "input":
            vals.append(np.asarray(inputs[node[1]]).astype(np.float64))
        elif k == "scalar":
            vals.append(np.float64(np.float32(scalars[node[1]])))
        elif k == "const":
            vals.append(np.float64(np.float32(node[2])))
        elif k == "iota":
            shp = [1] * spec.ndim; shp[node[1]] = full[node[1]]
            vals.append(np.arange(full[node[1]], dtype=np.float64).reshape(shp))
        elif k == "apply":
            a = [vals[i] for i in node[2]]
            if node[1] in _UN: vals.append(_UN[node[1]](a[0]))
            elif node[1] in _BIN: vals.append(_BIN[node[1]](a[0], a[1]))
            elif node[1] in _CMP: vals.append(_CMP[node[1]](a[0], a[1]).astype(np.float64))
            else: vals.append(np.where(a[0] != 0, a[1], a[2]))
        elif k == "reduce":
            fn = {"sum": np.sum, "max": np.max, "min": np.min, "prod": np.prod}[node[1]]
            vals.append(fn(np.asarray(vals[node[2]]), axis=node[3], keepdims=True)
                        if np.ndim(vals[node[2]]) else vals[node[2]])
        else:
            raise AssertionError(k)
    return vals


@pytest.mark.parametrize("seed", range(40))
def test_random_graphs_vs_numpy(oracle, seed):
    rng = np.random.default_rng(1000 + seed)
    ndim = int(rng.integers(1, 5))
    full = [int(rng.integers(1, 6)) for _ in range(ndim)]
    s = GraphSpec(ndim)
    inputs, vals = [], []
    for _ in range(int(rng.integers(1, 4))):
        bc = tuple(bool(rng.integers(0, 3) == 0) for _ in range(ndim))
        shp = [1 if b else e for b, e in zip(bc, full)]
        # a strided view: slice of a larger permuted base
        perm = rng.permutation(ndim)
        big = rng.uniform(0.2, 2.0, [2 * shp[p] + 1 for p in perm]).astype(np.float32)
        view = big.transpose(np.argsort(perm))[tuple(slice(1, 1 + 2 * e, 2) for e in shp)]
        assert list(view.shape) == shp
        inputs.append(view)
        vals.append(s.input("f32", bc))
    inputs[0] = np.ascontiguousarray(np.broadcast_to(inputs[0], full)) if False else inputs[0]
    sc = s.scalar("f32"); vals.append(sc)
    safe_un = ["neg", "abs", "exp", "log1p", "sqrt", "tanh", "sigmoid", "sqr", "recip", "expm1", "log"]
    for _ in range(int(rng.integers(2, 9))):
        r = rng.integers(0, 10)
        if r < 4:
            op = safe_un[int(rng.integers(len(safe_un)))]
            a = vals[int(rng.integers(len(vals)))]
            # keep arguments positive where the domain needs it
            v = s.apply(op, s.apply("abs", a) if op in ("log", "sqrt", "log1p", "recip") else a)
            if op in ("log", "recip"):
                v = s.apply(op, s.add(s.apply("abs", a), s.const(0.5)))
        elif r < 8:
            op = ["add", "sub", "mul", "max", "min"][int(rng.integers(5))]
            v = s.apply(op, vals[int(rng.integers(len(vals)))], vals[int(rng.integers(len(vals)))])
        elif r < 9:
            a, b, c = (vals[int(rng.integers(len(vals)))] for _ in range(3))
            v = s.apply("where", s.apply("gt", a, b), c, a)
        else:
            axes = tuple(sorted(set(int(x) for x in rng.integers(0, ndim, int(rng.integers(1, ndim + 1))))))
            v = s.reduce(["sum", "max", "min"][int(rng.integers(3))], vals[int(rng.integers(len(vals)))],
                         axes, keep=True)
        # tame growth so that float64-vs-float32-rounded comparisons stay meaningful
        v = s.apply("tanh", v) if rng.integers(0, 3) == 0 else v
        vals.append(v)
    s.output(vals[-1], "f32")
    s.output(vals[len(vals) // 2 + 1], "f32")
    scal = [float(rng.uniform(0.5, 1.5))]
    ref = _np_eval(s, inputs, scal, full)
    got = oracle.evaluate(s, inputs, scal)
    for (v, _), g in zip(s.outputs, got):
        want = np.asarray(ref[v], dtype=np.float64)
        want = want.reshape((1,) * (ndim - want.ndim) + want.shape) if want.ndim < ndim else want
        assert g.shape == want.shape, (g.shape, want.shape)
        with np.errstate(over="ignore"):
            assert np.allclose(g, want.astype(np.float32), rtol=2e-7, atol=0, equal_nan=True)


def test_no_nan_in_config_outputs(oracle):
    for w in (wl.c1_affine_tanh(16, 8), wl.c2_lstm_cell(4, 8), wl.c3_softmax_xent(5, 40),
              wl.c4_bias_relu_chansum(2, 3, 4, 5), wl.c5_stress(2, 3, 4, 5), wl.c5_stress(2, 3, 4, 5, "B")):
        for o in oracle.evaluate(w.spec, wl.host_inputs(w), w.scalars):
            assert np.isfinite(o.astype(np.float64)).all(), w.name


def test_threads_do_not_change_results(oracle):
    w = wl.c3_softmax_xent(37, 101)
    a = oracle.evaluate(w.spec, wl.host_inputs(w), nthreads=1)
    b = oracle.evaluate(w.spec, wl.host_inputs(w), nthreads=5)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


# ------------------------------------------------------------------ reductions: NaN order, int32, dropped axes

def _reduce_spec(red, storage, axes=(1,), keep=False, ndim=2, out=None):
    s = GraphSpec(ndim)
    v = s.reduce(red, s.input(storage, (False,) * ndim), axes, keep=keep)
    s.output(v, out or ("i32" if red == "argmax" or storage == "i32" else "f32"))
    return s


@pytest.mark.parametrize("where_nan", ["first", "middle", "last", "two", "all", "after_inf"])
def test_reduce_max_min_argmax_with_nan(oracle, where_nan):
    """max and min over an axis propagate NaN wherever it stands (numpy's max/min do the same);
    for arg-max a NaN ranks above every number, +inf included, and the first NaN wins (numpy's
    argmax has the same convention).  Rows without NaN sit beside the NaN rows."""
    nan, inf = np.float32("nan"), np.float32("inf")
    x = np.array([[3, 1, 4, 1, 5, 9, 2], [2, 7, 1, 8, 2, 8, 1], [-1, -2, -3, -1, -5, -6, -7]], np.float32)
    x = np.repeat(x[None], 2, 0).reshape(6, 7).copy()          # rows 3..5 stay free of NaN
    pos = {"first": [0], "middle": [3], "last": [6], "two": [2, 5], "all": list(range(7)), "after_inf": [4]}[where_nan]
    x[:3, pos] = nan
    if where_nan == "after_inf":
        x[:3, 1] = inf                                           # +inf before the NaN: the NaN still wins
    for red, fn in (("max", np.max), ("min", np.min)):
        got = oracle.evaluate(_reduce_spec(red, "f32"), [x])[0]
        with np.errstate(invalid="ignore"):
            want = fn(x, axis=1)
        assert np.isnan(got[:3]).all() and np.array_equal(got, want, equal_nan=True), red
        # the same along the other axis, through a transposed view
        got_t = oracle.evaluate(_reduce_spec(red, "f32", axes=(0,)), [x.T])[0]
        assert np.array_equal(got_t, want, equal_nan=True), red
    got = oracle.evaluate(_reduce_spec("argmax", "f32"), [x])[0]
    assert got.dtype == np.int32
    assert np.array_equal(got, np.argmax(x, axis=1))
    assert list(got[:3]) == [pos[0]] * 3
    assert list(got[3:]) == [5, 3, 0]                            # ties: the first of the two 8s, of the two -1s


def test_reduce_max_min_nan_through_an_expression(oracle):
    # the NaN is made by the expression under the reduction (0 * inf), not read from memory
    x = np.array([[1, 2, 3, 4], [1, np.inf, 3, 4], [5, 6, 7, np.inf]], np.float32)
    s = GraphSpec(2)
    v = s.mul(s.input("f32", (False, False)), s.const(0.0))
    s.output(s.reduce("max", v, (1,)), "f32"); s.output(s.reduce("argmax", v, (1,)), "i32")
    mx, am = oracle.evaluate(s, [x])
    assert np.array_equal(mx, np.float32([0, np.nan, np.nan]), equal_nan=True)
    assert list(am) == [0, 1, 3]


def test_int32_unary_ops_wrap_like_twos_complement(oracle):
    lo, hi = -2**31, 2**31 - 1
    a = np.array([lo, lo + 1, -46341, -46340, -7, -1, 0, 1, 7, 46340, 46341, 65536, hi - 1, hi], np.int32)
    with np.errstate(over="ignore"):
        want = {"neg": np.negative(a), "abs": np.abs(a), "sqr": a * a}
    # hand values for the corner cases (numpy wraps too, but these do not depend on it)
    assert want["neg"][0] == lo and want["abs"][0] == lo and want["sqr"][0] == 0
    assert want["sqr"][10] == np.int32(46341 * 46341 - 2**32) and want["sqr"][11] == 0
    assert want["sqr"][-1] == 1 and want["abs"][1] == hi and want["neg"][-1] == lo + 1
    for op in ("neg", "abs", "sqr"):
        got = oracle.evaluate(unary_spec(op, storage="i32", out="i32"), [a])[0]
        assert got.dtype == np.int32 and np.array_equal(got, want[op]), op


def test_int32_reductions_wrap_and_order(oracle):
    hi = 2**31 - 1
    a = np.array([[hi, 1, 5, -3], [hi, hi, hi, hi], [-2**31, -1, 0, 0], [65536, 65536, 3, 1],
                  [7, -2, 7, 3], [46341, 46341, 2, 1]], np.int32)
    with np.errstate(over="ignore"):
        want_sum = a.sum(axis=1, dtype=np.int32); want_prod = a.prod(axis=1, dtype=np.int32)
    # by hand: hi + 1 wraps to -2^31, then + 5 - 3; four times hi = -4 mod 2^32; 65536^2 = 2^32 = 0
    assert want_sum[0] == -2**31 + 2 and want_sum[1] == -4 and want_sum[2] == hi and want_prod[3] == 0
    assert want_prod[1] == 1                                     # (-1)^4 mod 2^32
    assert want_prod[5] == (46341 * 46341 * 2) % 2**32 == 9266
    for red, want in (("sum", want_sum), ("prod", want_prod), ("max", a.max(1)), ("min", a.min(1)),
                      ("argmax", a.argmax(1))):
        got = oracle.evaluate(_reduce_spec(red, "i32"), [a])[0]
        assert got.dtype == np.int32 and np.array_equal(got, want), red
        # column direction on the transposed view: same numbers
        got_t = oracle.evaluate(_reduce_spec(red, "i32", axes=(0,)), [a.T])[0]
        assert np.array_equal(got_t, want), red
    assert list(oracle.evaluate(_reduce_spec("argmax", "i32"), [a])[0]) == [0, 0, 2, 0, 0, 0]   # ties: first
    # over both axes at once, and a sum of an int32 expression (iota) that needs no memory
    with np.errstate(over="ignore"):
        assert oracle.evaluate(_reduce_spec("sum", "i32", axes=(0, 1)), [a])[0] == a.sum(dtype=np.int32)
    s = GraphSpec(2)
    x = s.input("i32", (False, False))
    s.output(s.reduce("sum", s.add(s.mul(s.iota(1), s.const(2**30, "i32")), s.mul(x, s.const(0, "i32"))), (1,)), "i32")
    # 2^30 * (0+1+2+3) = 6 * 2^30 = 2^32 + 2^31, which is -2^31 in 32 bits (the terms themselves are
    # 0, 2^30, -2^31 and -2^30 after wrapping; their wrapped running sums 0, 2^30, -2^30, -2^31)
    assert list(oracle.evaluate(s, [a])[0]) == [-2**31] * 6


def _np_shape_rule(spec, full):
    """Broadcast pattern and dropped axes per node, from the stated rule: a reduction makes its
    axes broadcastable and, without keep, dropped; a point-wise value is broadcastable where all
    operands are and drops what any operand dropped, as far as it is broadcastable there."""
    nd = spec.ndim
    bc, dr = [], []
    for node in spec.nodes:
        k = node[0]
        if k == "input": bc.append(set(d for d in range(nd) if node[3][d])); dr.append(set())
        elif k in ("scalar", "const"): bc.append(set(range(nd))); dr.append(set())
        elif k == "iota": bc.append(set(range(nd)) - {node[1]}); dr.append(set())
        elif k == "cast": bc.append(set(bc[node[1]])); dr.append(set(dr[node[1]]))
        elif k == "apply":
            b = set(range(nd)); u = set()
            for a in node[2]: b &= bc[a]; u |= dr[a]
            bc.append(b); dr.append(u & b)
        else:
            b = bc[node[2]] | set(node[3]); u = dr[node[2]] | (set() if node[4] else set(node[3]))
            bc.append(b); dr.append(u & b)
    return bc, dr


@pytest.mark.parametrize("seed", range(30))
def test_random_graphs_with_dropped_axes_vs_numpy(oracle, seed):
    """Reductions over one or several axes with and without keep inside random expressions: values
    against numpy float64 (kept dimensions), shapes against the rule written out above."""
    rng = np.random.default_rng(5000 + seed)
    ndim = int(rng.integers(2, 5))
    full = [int(rng.integers(2, 5)) for _ in range(ndim)]
    s = GraphSpec(ndim)
    inputs, vals = [], []
    for k in range(int(rng.integers(1, 4))):
        bc = tuple(bool(k > 0 and rng.integers(0, 3) == 0) for _ in range(ndim))
        shp = [1 if b else e for b, e in zip(bc, full)]
        inputs.append(rng.uniform(0.5, 1.5, shp).astype(np.float32))
        vals.append(s.input("f32", bc))
    n_red = 0
    for _ in range(int(rng.integers(3, 8))):
        r = rng.integers(0, 10)
        if r < 5 or n_red >= 3:
            op = ["add", "sub", "mul", "max", "min"][int(rng.integers(5))]
            v = s.apply(op, vals[int(rng.integers(len(vals)))], vals[int(rng.integers(len(vals)))])
        else:
            axes = tuple(sorted(set(int(x) for x in rng.integers(0, ndim, int(rng.integers(1, ndim + 1))))))
            red = ["sum", "max", "min", "prod"][int(rng.integers(4))]
            v = s.reduce(red, vals[int(rng.integers(len(vals)))], axes, keep=bool(rng.integers(0, 2)))
            n_red += 1
        vals.append(v)
    outs = [vals[-1], vals[-2], vals[len(vals) // 2]]
    for v in outs:
        s.output(v, "f32")
    ref = _np_eval(s, inputs, [], full)
    bc, dr = _np_shape_rule(s, full)
    got = oracle.evaluate(s, inputs)
    for v, g in zip(outs, got):
        want = np.asarray(ref[v], dtype=np.float64)
        want = want.reshape((1,) * (ndim - want.ndim) + want.shape)
        want = np.broadcast_to(want, [1 if d in bc[v] else full[d] for d in range(ndim)])
        want = want.reshape([want.shape[d] for d in range(ndim) if d not in dr[v]])
        assert g.shape == want.shape, (g.shape, want.shape, sorted(dr[v]))
        assert np.allclose(g, want.astype(np.float32), rtol=3e-7, atol=0)


def test_multi_axis_reductions_without_keep_have_the_rank_of_the_kept_axes(oracle):
    rng = np.random.default_rng(77)
    X = rng.integers(-4, 5, (3, 4, 5, 2)).astype(np.float32)
    for axes in [(0, 1), (1, 3), (0, 2, 3), (0, 1, 2, 3), (2,)]:
        for red, fn in (("sum", np.sum), ("max", np.max), ("min", np.min), ("prod", np.prod)):
            got = oracle.evaluate(_reduce_spec(red, "f32", axes=axes, keep=False, ndim=4), [X])[0]
            want = fn(X.astype(np.float64), axis=axes)
            assert got.shape == want.shape and np.array_equal(got, want), (red, axes)
    # a value computed from two reductions: an axis dropped by either stays dropped where the
    # result is constant along it, and comes back where the other operand varies along it
    s = GraphSpec(3)
    x = s.input("f32", (False, False, False))
    a = s.reduce("sum", x, (0, 2), keep=False); b = s.reduce("max", x, (2,), keep=False); c = s.reduce("sum", x, (0,), keep=True)
    s.output(s.mul(a, b), "f32"); s.output(s.add(a, c), "f32"); s.output(s.add(a, x), "f32")
    Y = rng.integers(-3, 4, (2, 3, 4)).astype(np.float32); Y64 = Y.astype(np.float64)
    ab, ac, ax = oracle.evaluate(s, [Y])
    assert ab.shape == (2, 3) and np.array_equal(ab, Y64.sum((0, 2))[None, :] * Y64.max(2))
    # axis 0: dropped by a, kept (as extent 1) by c, constant in the sum -> stays dropped
    assert ac.shape == (3, 4) and np.array_equal(ac, (Y64.sum((0, 2), keepdims=True) + Y64.sum(0, keepdims=True))[0])
    assert ax.shape == (2, 3, 4) and np.array_equal(ax, Y64.sum((0, 2), keepdims=True) + Y64)


# Arg-max over several axes: the position of the first maximum in the row-major order of the
# reduced axes, in axis order (what numpy gives after moving those axes last and flattening them).
@pytest.mark.parametrize("axes", [(0, 1), (1, 2), (0, 2), (0, 1, 2), (2,), (0, 3), (1, 2, 3)])
@pytest.mark.parametrize("keep", [False, True])
def test_argmax_over_several_axes_vs_numpy(oracle, axes, keep):
    rng = np.random.default_rng(77 + sum(axes))
    shape = (3, 4, 5, 2)
    x = rng.integers(-3, 4, shape).astype(np.float32)          # few distinct values: many ties
    x[1, 2, 3, 0] = np.nan
    x[2, 0, 0, 1] = np.nan
    s = GraphSpec(4)
    xi = s.input("f32", (False,) * 4)
    s.output(s.reduce("argmax", xi, axes, keep=keep), "i32")
    s.output(s.reduce("max", xi, axes, keep=keep), "f32")
    got, mx = oracle.evaluate(s, [x])
    kept = [d for d in range(4) if d not in axes]
    moved = np.transpose(x, kept + list(axes)).reshape([shape[d] for d in kept] + [-1])
    want = np.argmax(moved, axis=-1)                            # numpy: first occurrence, NaN counts as the maximum
    if keep:
        want = want.reshape([1 if d in axes else shape[d] for d in range(4)])
    assert got.shape == want.shape and np.array_equal(got, want)
    # and the value found there is the maximum
    flat_max = np.take_along_axis(moved, np.argmax(moved, axis=-1)[..., None], axis=-1)[..., 0]
    assert np.array_equal(mx.reshape(flat_max.shape), flat_max, equal_nan=True)


def test_argmax_over_two_axes_by_hand(oracle):
    x = np.array([[[1, 9], [9, 2]], [[3, 3], [3, 3]]], np.float32)      # [2, 2, 2]
    s = GraphSpec(3)
    xi = s.input("f32", (False,) * 3)
    s.output(s.reduce("argmax", xi, (1, 2)), "i32")         # per leading index: positions in a 2 x 2 block
    s.output(s.reduce("argmax", xi, (0, 2)), "i32")         # per middle index: positions in [2 (axis 0), 2 (axis 2)]
    a12, a02 = oracle.evaluate(s, [x])
    assert a12.tolist() == [1, 0]                           # 9 first at (0, 1) -> 1; all equal -> 0
    assert a02.tolist() == [1, 0]                           # middle 0: values 1 9 3 3 -> 1; middle 1: 9 2 3 3 -> 0


def test_run_time_scalars_have_their_declared_type(oracle):
    # a float32 scalar is rounded to float32 before use, an int32 scalar is truncated toward zero
    x = np.array([[1.0, 2.0, 4.0]], np.float32)
    k = np.array([[3, -3, 10]], np.int32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); ki = s.input("i32", (False, False))
    a = s.scalar("f32"); n = s.scalar("i32")
    s.output(s.mul(xi, a), "f32")
    s.output(s.add(ki, n), "i32")
    s.output(s.mul(s.cast(n, "f32"), xi), "f32")
    s.output(s.add(s.mul(xi, s.const(0.0)), s.sub(a, s.const(16777216.0))), "f32")
    got = oracle.evaluate(s, [x, k], [0.1, 7.9])
    assert np.array_equal(got[0], (x.astype(np.float64) * np.float64(np.float32(0.1))).astype(np.float32))
    assert got[1].tolist() == [[10, 4, 17]]
    assert got[2].tolist() == [[7.0, 14.0, 28.0]]
    got = oracle.evaluate(s, [x, k], [-2.5, -7.9])
    assert got[0].tolist() == [[-2.5, -5.0, -10.0]] and got[1].tolist() == [[-4, -10, 3]] and got[2].tolist() == [[-7.0, -14.0, -28.0]]
    # 2^24 + 1 is not a float32: the scalar is 2^24 by the time it is used
    got = oracle.evaluate(s, [x, k], [16777217.0, 0.0])
    assert got[3].tolist() == [[0.0, 0.0, 0.0]]
