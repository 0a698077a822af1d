"""GPU parity, part 2: every scalar operation on its own, and randomly generated graphs over
random shapes, broadcast patterns and strided views -- all against the CPU oracle on the same
seeded inputs.  Launches go through the C ABI binding."""
import numpy as np
import pytest

from workloads import GraphSpec

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def G():
    import torch
    import tests.harness as h
    from paper_1605_02688_amd import ewf

    class Ctx:
        pass
    c = Ctx()
    c.torch, c.h, c.ewf = torch, h, ewf
    return c


def run_spec(G, spec, host_inputs, scalars=(), **opts):
    """host_inputs: numpy arrays (possibly strided views).  The device tensors reproduce the
    same strides over a copy of each view's underlying buffer."""
    torch = G.torch
    dev = []
    for a in host_inputs:
        base = a if a.base is None else a.base
        while base.base is not None:
            base = base.base
        tb = torch.from_numpy(np.ascontiguousarray(base).reshape(-1).copy()).cuda()
        off = (a.__array_interface__["data"][0] - base.__array_interface__["data"][0]) // a.itemsize
        dev.append(torch.as_strided(tb, a.shape, tuple(s // a.itemsize for s in a.strides), off))
    expr = G.ewf.Expression(spec, **opts)
    outs = G.h.alloc_outputs(expr, spec, dev)
    ws = G.h.make_workspace(expr, dev, outs)
    expr.run(dev, outs, scalars, ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return expr, [o.cpu().numpy() for o in outs]


# ------------------------------------------------------------------ single operations

UNARY = {
    # name: (low, high, rtol, atol) -- float32 element-wise bar unless the op amplifies input error
    "neg": (-4, 4, 0, 0), "abs": (-4, 4, 0, 0), "sqr": (-4, 4, 2e-6, 1e-6), "exp": (-20, 20, 2e-6, 1e-6),
    "log": (1e-3, 50, 2e-6, 1e-6), "log1p": (-0.9, 50, 2e-6, 1e-6), "sqrt": (0, 50, 2e-6, 1e-6),
    "tanh": (-12, 12, 2e-6, 1e-6), "sigmoid": (-30, 30, 2e-6, 1e-6), "expm1": (-10, 10, 2e-6, 1e-6),
    "recip": (0.05, 50, 2e-6, 1e-6),
}


@pytest.mark.parametrize("op", sorted(UNARY))
def test_unary_op_accurate_mode(op, oracle, G):
    lo, hi, rtol, atol = UNARY[op]
    rng = np.random.default_rng(hash(op) % 1000)
    x = rng.uniform(lo, hi, 5003).astype(np.float32)
    x[:7] = np.float32([lo, hi, (lo + hi) / 2, lo + 1e-4, hi - 1e-4, lo + 1e-7 * (hi - lo), 1.0])
    s = GraphSpec(1)
    s.output(s.apply(op, s.input("f32", (False,))), "f32")
    print(f"[case] unary {op}", flush=True)
    _, (got,) = run_spec(G, s, [x])
    want = oracle.evaluate(s, [x])[0]
    G.h.compare(op, got, want, rtol, atol)


def test_exp_accurate_mode_whole_range(oracle, G):
    # the accurate exp is the library's own (hardware exp2 plus a first-order correction):
    # a few units in the last place from underflow to overflow, exact at the special values
    rng = np.random.default_rng(77)
    x = np.concatenate([rng.uniform(-87.3, 88.7, 200000), np.linspace(-87.3, 88.7, 50001),
                        rng.uniform(-1e-3, 1e-3, 1000)]).astype(np.float32)
    sp = np.float32([0.0, -0.0, np.inf, -np.inf, np.nan, 88.8, 100.0, 1e30, -104.0, -1e30, 1e-40, 88.72283,
                     3.0e38, -3.0e38, -3.4028235e38, 3.4028235e38])          # x * log2(e) overflows for the last four
    x = np.concatenate([sp, x])
    s = GraphSpec(1)
    s.output(s.apply("exp", s.input("f32", (False,))), "f32")
    expr, (got,) = run_spec(G, s, [x], math_mode=1)
    assert "ewf_acc::exp" in expr.source()
    want = oracle.evaluate(s, [x])[0]
    k = len(sp)
    with np.errstate(over="ignore", invalid="ignore"):
        assert got[0] == 1.0 and got[1] == 1.0 and got[2] == np.inf and got[3] == 0.0 and np.isnan(got[4])
        assert np.all(got[5:8] == np.inf) and np.all(got[8:10] == 0.0) and got[10] == 1.0
        assert got[12] == np.inf and got[13] == 0.0 and got[14] == 0.0 and got[15] == np.inf
    G.h.compare("exp", got[k:], want[k:], 4e-7, 0)          # about three units in the last place


def test_tanh_and_sigmoid_accurate_mode_whole_range(oracle, G):
    # the library's own routines (hardware exp2 and reciprocal, a series near 0): a few units
    # in the last place everywhere, exact at the special values
    rng = np.random.default_rng(78)
    x = np.concatenate([rng.uniform(-1, 1, 200000), rng.uniform(-20, 20, 100000), np.linspace(-0.3, 0.3, 60001),
                        rng.uniform(-100, 100, 20000), rng.uniform(-1e-4, 1e-4, 2000)]).astype(np.float32)
    sp = np.float32([0.0, -0.0, np.inf, -np.inf, np.nan, 1e30, -1e30, 44.0, 88.0, -88.0, 89.0, -104.0, 1e-30, -1e-38])
    x = np.concatenate([sp, x])
    s = GraphSpec(1)
    xi = s.input("f32", (False,))
    s.output(s.apply("tanh", xi), "f32"); s.output(s.apply("sigmoid", xi), "f32")
    expr, (gt, gs) = run_spec(G, s, [x], math_mode=1)
    assert "ewf_acc::tanh" in expr.source() and "ewf_acc::sigmoid" in expr.source()
    wt, ws = oracle.evaluate(s, [x])
    k = len(sp)
    assert gt[0] == 0 and not np.signbit(gt[0]) and gt[1] == 0 and np.signbit(gt[1])
    assert gt[2] == 1 and gt[3] == -1 and np.isnan(gt[4]) and gt[5] == 1 and gt[6] == -1
    assert gs[0] == 0.5 and gs[2] == 1 and gs[3] == 0 and np.isnan(gs[4]) and gs[5] == 1 and gs[6] == 0
    G.h.compare("tanh", gt[k:], wt[k:], 6e-7, 0)            # ten units in the last place at most
    G.h.compare("tanh specials", gt[:k], wt[:k], 6e-7, 0)
    G.h.compare("sigmoid", gs[k:], ws[k:], 4e-7, 1.2e-38)   # results below the smallest normal may flush
    G.h.compare("sigmoid specials", gs[:k], ws[:k], 4e-7, 1.2e-38)


def test_tanh_and_sigmoid_automatic_mode_whole_range(oracle, G):
    # under the automatic math mode float32 results take the native-rate sigmoid and tanh: held to
    # the element-wise bar over the whole range, dense around the switch to the series of tanh
    # (|x| = 2^-5) and where the exponential's argument is large, alone and as factors of a product
    rng = np.random.default_rng(79)
    x = np.concatenate([rng.uniform(-1, 1, 200000), rng.uniform(-20, 20, 100000), np.linspace(-0.3, 0.3, 60001),
                        np.linspace(0.03, 0.0325, 20001), -np.linspace(0.03, 0.0325, 20001),
                        rng.uniform(-100, 100, 20000), rng.uniform(-1e-4, 1e-4, 2000)]).astype(np.float32)
    sp = np.float32([0.0, -0.0, np.inf, -np.inf, np.nan, 1e30, -1e30, 15.0, -15.0, 88.0, -88.0, 89.0, -104.0, 1e-30, -1e-38])
    x = np.concatenate([sp, x])
    y = rng.uniform(-3, 3, x.shape).astype(np.float32)
    s = GraphSpec(1)
    xi = s.input("f32", (False,)); yi = s.input("f32", (False,))
    t = s.apply("tanh", xi); g = s.apply("sigmoid", xi)
    s.output(t, "f32"); s.output(g, "f32")
    s.output(s.add(s.mul(g, yi), s.mul(s.apply("sigmoid", yi), t)), "f32")        # f * c + i * g of an LSTM cell
    expr, (gt, gs, gc) = run_spec(G, s, [x, y])
    assert "ewf_fast::tanh" in expr.source() and "ewf_fast::sigmoid" in expr.source()
    wt, ws, wc = oracle.evaluate(s, [x, y])
    assert gt[2] == 1 and gt[3] == -1 and np.isnan(gt[4]) and gs[2] == 1 and gs[3] == 0 and np.isnan(gs[4])
    G.h.compare("tanh", gt, wt, 2e-6, 1e-6)
    G.h.compare("sigmoid", gs, ws, 2e-6, 1e-6)
    terms = np.nan_to_num(np.abs(ws.astype(np.float64) * y) + np.abs(wt.astype(np.float64)), nan=0.0, posinf=0.0)
    G.h.compare("cell", gc, wc, 2e-6, 1e-6, scale=np.maximum(terms, np.abs(np.where(np.isfinite(wc), wc, 0.0))))
    # the relative error alone, away from the flush to zero of tiny sigmoids: under 1.5e-6 as stated
    fin = np.isfinite(wt) & (wt != 0)
    assert np.max(np.abs(gt[fin].astype(np.float64) - wt[fin]) / np.abs(wt[fin])) < 1.5e-6
    big = np.isfinite(ws) & (ws > 1e-30)
    assert np.max(np.abs(gs[big].astype(np.float64) - ws[big]) / ws[big]) < 1.5e-5     # exp of up to -69: |x| * 6e-8


def test_run_time_scalars_of_both_types(oracle, G):
    rng = np.random.default_rng(81)
    x = rng.standard_normal((37, 1003)).astype(np.float32)
    k = rng.integers(-100, 100, (37, 1003)).astype(np.int32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); ki = s.input("i32", (False, False))
    a = s.scalar("f32"); n = s.scalar("i32")
    s.output(s.mul(xi, a), "f32")
    s.output(s.add(ki, n), "i32")
    s.output(s.mul(s.cast(n, "f32"), xi), "f32")
    s.output(s.reduce("sum", s.apply("where", s.apply("gt", ki, n), xi, s.const(0.0)), (1,)), "f32")
    for scal in ([0.1, 7.9], [-2.5, -7.9], [16777217.0, 0.0]):
        expr, got = run_spec(G, s, [x, k], scal)
        want = oracle.evaluate(s, [x, k], scal)
        G.h.compare("x*a", got[0], want[0], 2e-6, 1e-6)
        assert np.array_equal(got[1], want[1])
        G.h.compare("n*x", got[2], want[2], 2e-6, 1e-6)
        G.h.compare("sum", got[3], want[3], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64)).sum(1))


def test_log1p_keeps_small_arguments(oracle, G):
    x = np.float32([1e-7, -1e-7, 3e-10, 1e-5, -1e-5])
    s = GraphSpec(1)
    s.output(s.apply("log1p", s.input("f32", (False,))), "f32")
    for mode in (1, 2):
        _, (got,) = run_spec(G, s, [x], math_mode=mode)
        assert np.allclose(got, x.astype(np.float64), rtol=1e-4), mode   # log(1+x) in float32 would give 0


BINARY = ["add", "sub", "mul", "div", "max", "min", "pow"]


@pytest.mark.parametrize("op", BINARY)
def test_binary_op_accurate_mode(op, oracle, G):
    rng = np.random.default_rng(5 + len(op))
    a = rng.uniform(-3, 3, 4099).astype(np.float32)
    b = rng.uniform(-3, 3, 4099).astype(np.float32)
    if op == "pow":
        a = np.abs(a) + np.float32(0.1)
    if op == "div":
        b = np.where(np.abs(b) < 0.05, np.float32(0.5), b)
    s = GraphSpec(1)
    s.output(s.apply(op, s.input("f32", (False,)), s.input("f32", (False,))), "f32")
    print(f"[case] binary {op}", flush=True)
    _, (got,) = run_spec(G, s, [a, b])
    want = oracle.evaluate(s, [a, b])[0]
    G.h.compare(op, got, want, 2e-6, 1e-6)


def test_compare_where_and_int_ops_are_exact(oracle, G):
    rng = np.random.default_rng(9)
    a = rng.integers(-3, 3, 1000).astype(np.float32); b = rng.integers(-3, 3, 1000).astype(np.float32)
    ia = rng.integers(-2**31, 2**31 - 1, 1000).astype(np.int32); ib = rng.integers(-70000, 70000, 1000).astype(np.int32)
    s = GraphSpec(1)
    x = s.input("f32", (False,)); y = s.input("f32", (False,))
    i = s.input("i32", (False,)); j = s.input("i32", (False,))
    for op in ("gt", "ge", "lt", "le", "eq", "ne"):
        s.output(s.apply(op, x, y), "i32")
        s.output(s.apply("where", s.apply(op, i, j), x, y), "f32")
    for op in ("add", "sub", "mul", "max", "min"):
        s.output(s.apply(op, i, j), "i32")
    s.output(s.apply("neg", i), "i32"); s.output(s.apply("abs", j), "i32"); s.output(s.apply("sqr", j), "i32")
    s.output(s.add(s.mul(s.iota(0), s.const(3, "i32")), j), "i32")
    s.output(s.cast(i, "f32"), "f32")
    s.output(s.cast(s.mul(x, s.const(1.75)), "i32"), "i32")
    s.output(s.cast(s.mul(x, s.const(0.3333)), "f16"), "f32")
    _, got = run_spec(G, s, [a, b, ia, ib])
    want = oracle.evaluate(s, [a, b, ia, ib])
    for k, (g_, w_) in enumerate(zip(got, want)):
        G.h.compare(f"out{k}", g_, w_, 0, 0)


def test_nan_and_inf_conventions(oracle, G):
    nan, inf = np.float32("nan"), np.float32("inf")
    a = np.float32([1, nan, 3, nan, inf, -inf, 0.0, -0.0]); b = np.float32([2, 2, nan, nan, 1, 1, nan, 5])
    s = GraphSpec(1)
    x = s.input("f32", (False,)); y = s.input("f32", (False,))
    s.output(s.apply("max", x, y), "f32"); s.output(s.apply("min", x, y), "f32")
    s.output(s.apply("where", x, y, s.const(7.0)), "f32")
    _, got = run_spec(G, s, [a, b])
    want = oracle.evaluate(s, [a, b])
    for g_, w_ in zip(got, want):
        assert np.array_equal(g_, w_, equal_nan=True)


def test_f16_storage_rounds_to_nearest_even(oracle, G):
    rng = np.random.default_rng(10)
    a = rng.uniform(-2, 2, 4096).astype(np.float16); b = rng.uniform(-2, 2, 4096).astype(np.float16)
    s = GraphSpec(1)
    s.output(s.mul(s.input("f16", (False,)), s.input("f16", (False,))), "f16")
    _, (got,) = run_spec(G, s, [a, b])
    # the product of two float16 values is exact in float32, so the stored result is the
    # correctly rounded one: bit-exact against the oracle
    assert np.array_equal(got, oracle.evaluate(s, [a, b])[0])


def test_native_rate_math_meets_the_f16_bar(oracle, G):
    rng = np.random.default_rng(11)
    x = rng.uniform(-6, 6, 20000).astype(np.float16)
    p = rng.uniform(0.1, 5, 20000).astype(np.float16)
    s = GraphSpec(1)
    a = s.input("f16", (False,)); b = s.input("f16", (False,))
    for op in ("exp", "tanh", "sigmoid", "expm1"):
        s.output(s.apply(op, a), "f16")
    for op in ("log", "log1p", "sqrt", "recip"):
        s.output(s.apply(op, b), "f16")
    s.output(s.apply("pow", b, s.mul(a, s.const(0.25))), "f16")
    s.output(s.div(a, b), "f16")
    want = oracle.evaluate(s, [x, p])
    for mode, flavour in ((0, "ewf_bare::"), (2, "ewf_fast::"), (3, "ewf_bare::")):
        expr, got = run_spec(G, s, [x, p], math_mode=mode)
        assert flavour in expr.source()
        for k, (g_, w_) in enumerate(zip(got, want)):
            G.h.compare(f"mode{mode}.out{k}", g_, w_, 2e-3, 1e-3)


def test_run_time_scalars_reach_every_stage_of_a_plan(oracle, G):
    # a temperature and an offset, used before and after the reductions of a plan in several kernels
    rng = np.random.default_rng(82)
    x = rng.standard_normal((40, 70001)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    t = s.scalar("f32"); off = s.scalar("f32"); n = s.scalar("i32")
    z = s.mul(xi, t)
    m = s.reduce("max", z, (1,), keep=True)
    S = s.reduce("sum", s.apply("exp", s.sub(z, m)), (1,), keep=True)
    lse = s.add(s.add(m, s.apply("log", S)), off)
    s.output(lse, "f32")
    s.output(s.div(s.apply("exp", s.sub(z, m)), S), "f32")                      # probabilities: a second sweep
    s.output(s.mul(s.reduce("sum", lse, (0, 1)), s.cast(n, "f32")), "f32")     # over the rows, times an integer scalar
    for scal in ([0.5, 3.0, 2.0], [2.0, -1.0, -3.0]):
        expr, got = run_spec(G, s, [x], scal)
        info = expr.info()
        assert info["kernel_class"] == "multi" and info["grid_blocks"] >= 2, info
        want = oracle.evaluate(s, [x], scal)
        G.h.compare("lse", got[0], want[0], 1e-5, 1e-6)
        G.h.compare("p", got[1], want[1], 1e-5, 1e-9)
        G.h.compare("total", got[2], want[2], 1e-5, 1e-6, scale=np.abs(want[0].astype(np.float64)).sum() * abs(scal[2]))


def test_every_operation_folds_on_literals_like_it_evaluates(oracle, G):
    # op(literal, literal) is folded on the host when an expression is compiled; the oracle
    # evaluates it like any other node.  Every operation, float32 and int32, special values included.
    x = np.linspace(-1, 1, 513).astype(np.float32)
    k = np.arange(513, dtype=np.int32)
    fl = [(0.75, 1.5), (-2.25, 0.5), (3.0, -1.25), (0.0, 2.0), (1e-3, 1e-3)]
    unary = ["neg", "abs", "sqr", "exp", "tanh", "sigmoid", "recip", "expm1"]
    positive = ["log", "log1p", "sqrt"]
    binary = ["add", "sub", "mul", "div", "max", "min"]
    compare = ["gt", "ge", "lt", "le", "eq", "ne"]
    for a, b in fl:
        s = GraphSpec(1)
        xi = s.input("f32", (False,)); ki = s.input("i32", (False,))
        zero = s.mul(xi, s.const(0.0))
        izero = s.mul(ki, s.const(0, "i32"))
        ca, cb = s.const(a), s.const(b)
        vals = [s.apply(op, ca) for op in unary] + [s.apply(op, s.apply("abs", ca)) for op in positive]
        vals += [s.apply(op, ca, cb) for op in binary] + [s.apply("pow", s.apply("abs", ca), cb)]
        vals += [s.apply("where", s.apply(op, ca, cb), ca, cb) for op in compare]
        total = zero
        for v in vals:
            total = s.add(total, v)
        s.output(total, "f32")
        for v in vals[:6]:
            s.output(s.add(zero, v), "f32")
        ia, ib = s.const(int(a * 4), "i32"), s.const(int(b * 4) - 7, "i32")
        ivals = [s.apply(op, ia) for op in ("neg", "abs", "sqr")] + [s.apply(op, ia, ib) for op in ("add", "sub", "mul", "max", "min")]
        ivals += [s.apply("where", s.apply(op, ia, ib), ia, ib) for op in compare]
        ivals += [s.cast(s.mul(ca, s.const(3.7)), "i32"), s.mul(s.const(46341, "i32"), s.const(46341, "i32"))]
        itotal = izero
        for v in ivals:
            itotal = s.add(itotal, v)
        s.output(itotal, "i32")
        s.output(s.add(zero, s.cast(s.cast(cb, "f16"), "f32")), "f32")
        expr, got = run_spec(G, s, [x, k])
        before, after = expr.graph_size()
        assert after <= before - 30, (before, after)          # the operations on literals are gone (the sums of them stay)
        want = oracle.evaluate(s, [x, k])
        terms = len(vals)
        G.h.compare(f"sum of folds {a},{b}", got[0], want[0], 2e-6 * terms, 1e-6 * terms)
        for i in range(1, 7):
            G.h.compare(f"fold {i} {a},{b}", got[i], want[i], 2e-6, 1e-6)
        assert np.array_equal(got[7], want[7]), (a, b, got[7][:3], want[7][:3])
        assert np.array_equal(got[8], want[8])


def test_rewritten_graph_matches_the_graph_as_described(oracle, G):
    # the oracle evaluates the description node by node; the library first merges duplicates,
    # folds constants and applies the stabilising rewrites
    rng = np.random.default_rng(185)
    x = rng.uniform(-3, 3, 6000).astype(np.float32)
    x[:6] = np.float32([1e-7, -1e-7, 3e-10, 0.0, 20.0, -20.0])
    y = rng.uniform(0.1, 2, 6000).astype(np.float32)
    s = GraphSpec(1)
    xi = s.input("f32", (False,)); yi = s.input("f32", (False,))
    softplus = s.apply("log", s.add(s.const(1.0), s.apply("exp", xi)))                 # -> log1p(exp(x))
    em1 = s.sub(s.apply("exp", xi), s.const(1.0))                                     # -> expm1(x)
    sq = s.apply("pow", s.add(s.mul(yi, s.const(1.0)), s.const(0.0)), s.const(2.0))   # -> y * y
    k = s.apply("exp", s.mul(s.const(0.5), s.const(-2.0)))                            # -> literal e^-1
    dup = s.apply("tanh", s.mul(xi, yi)); dup2 = s.apply("tanh", s.mul(yi, xi))       # one node
    s.output(softplus, "f32"); s.output(em1, "f32"); s.output(sq, "f32")
    s.output(s.mul(s.add(dup, dup2), k), "f32")
    want = oracle.evaluate(s, [x, y])
    for opts in ({}, {"no_rewrite": 1}):
        expr, got = run_spec(G, s, [x, y], **opts)
        before, after = expr.graph_size()
        assert (after < before) == (not opts)
        for k_, (g_, w_) in enumerate(zip(got, want)):
            if opts and k_ == 1:
                # exp(x) - 1 as described loses the small arguments in float32; only the rewritten form meets the bar there
                G.h.compare(f"described.out{k_}", g_[6:], w_[6:], 2e-6, 1e-6)
                continue
            G.h.compare(f"{'described' if opts else 'rewritten'}.out{k_}", g_, w_, 2e-6, 1e-6)
    # the stable forms keep the tiny arguments that the described forms would lose
    expr, got = run_spec(G, s, [x, y])
    assert np.allclose(got[1][:3], x[:3].astype(np.float64), rtol=1e-5)


# ------------------------------------------------------------------ layouts

def test_transpose_and_slice_views(oracle, G):
    rng = np.random.default_rng(12)
    base = rng.standard_normal((70, 90)).astype(np.float32)
    s = GraphSpec(2)
    s.output(s.apply("tanh", s.add(s.input("f32", (False, False)), s.input("f32", (False, False)))), "f32")
    for a, b in [(base[:64, :64], base[3:67, 5:69].T), (base[1:60:2, ::3], base[:30, :30]),
                 (base.T[:33, :17], base[:33, 20:37])]:
        _, (got,) = run_spec(G, s, [a, b])
        want = oracle.evaluate(s, [a, b])[0]
        G.h.compare("views", got, want, 2e-6, 1e-6)
        # a strided view gives exactly what its contiguous copy gives
        _, (got2,) = run_spec(G, s, [np.ascontiguousarray(a), np.ascontiguousarray(b)])
        assert np.array_equal(got, got2)


def test_broadcast_equals_materialised_operand(oracle, G):
    rng = np.random.default_rng(13)
    X = rng.standard_normal((9, 33, 20)).astype(np.float32)
    b = rng.standard_normal((1, 33, 1)).astype(np.float32)
    s = GraphSpec(3)
    s.output(s.apply("exp", s.mul(s.input("f32", (False,) * 3), s.input("f32", (True, False, True)))), "f32")
    s2 = GraphSpec(3)
    s2.output(s2.apply("exp", s2.mul(s2.input("f32", (False,) * 3), s2.input("f32", (False,) * 3))), "f32")
    _, (g1,) = run_spec(G, s, [X, b])
    _, (g2,) = run_spec(G, s2, [X, np.ascontiguousarray(np.broadcast_to(b, X.shape))])
    assert np.array_equal(g1, g2)


def test_in_place_output(oracle, G):
    torch = G.torch
    rng = np.random.default_rng(14)
    x = rng.standard_normal((300, 77)).astype(np.float32)
    s = GraphSpec(2)
    s.output(s.apply("sigmoid", s.input("f32", (False, False))), "f32")
    want = oracle.evaluate(s, [x])[0]
    t = torch.from_numpy(x.copy()).cuda()
    expr = G.ewf.Expression(s)
    expr.run([t], [t], (), None, torch.cuda.current_stream().cuda_stream)      # overwrites its input
    torch.cuda.synchronize()
    G.h.compare("inplace", t.cpu().numpy(), want, 2e-6, 1e-6)
    u = torch.zeros(301, 77, device="cuda")
    with pytest.raises(G.ewf.EwfError) as e:                                    # shifted overlap is refused
        expr.run([u[:300]], [u[1:]], (), None, 0)
    assert e.value.status == G.ewf.EALIAS


def test_index64_kernels_give_the_same_result(oracle, G):
    rng = np.random.default_rng(15)
    x = rng.standard_normal((50, 70)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    s.output(s.apply("tanh", xi), "f32"); s.output(s.reduce("sum", xi, (1,)), "f32")
    e32, g32 = run_spec(G, s, [x])
    e64, g64 = run_spec(G, s, [x], force_index64=1)
    assert e64.info()["index_bits"] == 64 and e32.info()["index_bits"] == 32
    for a, b in zip(g32, g64):
        assert np.array_equal(a, b)


def test_canary_around_outputs(oracle, G):
    # outputs live in the middle of a larger buffer; nothing outside the view may change
    torch = G.torch
    rng = np.random.default_rng(16)
    x = rng.standard_normal((37, 53)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    s.output(s.apply("exp", xi), "f32"); s.output(s.reduce("max", xi, (1,)), "f32")
    expr = G.ewf.Expression(s)
    big = torch.full((45, 64), -777.0, device="cuda")
    big2 = torch.full((64,), -777.0, device="cuda")
    out = big[4:41, 5:58]; red = big2[9:46]
    t = torch.from_numpy(x).cuda()
    ws = G.h.make_workspace(expr, [t], [out, red])
    expr.run([t], [out, red], (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = oracle.evaluate(s, [x])
    G.h.compare("exp", out.cpu().numpy(), want[0], 2e-6, 1e-6)
    G.h.compare("max", red.cpu().numpy(), want[1], 0, 0)
    mask = torch.ones_like(big, dtype=torch.bool); mask[4:41, 5:58] = False
    assert bool((big[mask] == -777.0).all())
    mask2 = torch.ones_like(big2, dtype=torch.bool); mask2[9:46] = False
    assert bool((big2[mask2] == -777.0).all())


# ------------------------------------------------------------------ reductions

def test_integer_valued_sums_are_bit_exact(oracle, G):
    # |sum| < 2^24 and integer-valued data: every association order gives the same float32
    rng = np.random.default_rng(17)
    for shape, axes in [((64, 1000), (1,)), ((300, 40), (1,)), ((3, 7, 3000), (0, 2)), ((100000,), (0,)),
                        ((5, 33, 21, 40), (0, 2, 3)), ((2, 70000), (1,))]:
        X = rng.integers(-20, 20, shape).astype(np.float32)
        s = GraphSpec(len(shape))
        s.output(s.reduce("sum", s.input("f32", (False,) * len(shape)), axes), "f32")
        print(f"[case] exact sum {shape} axes {axes}", flush=True)
        expr, (got,) = run_spec(G, s, [X])
        assert np.array_equal(got, X.astype(np.float64).sum(axis=axes).astype(np.float32)), (shape, expr.info())
        assert np.array_equal(got, oracle.evaluate(s, [X])[0])


def test_reductions_over_an_empty_axis_give_the_identity(oracle, G):
    import torch
    x = np.zeros((5, 0, 3), np.float32)
    s = GraphSpec(3)
    xi = s.input("f32", (False,) * 3)
    s.output(s.reduce("sum", xi, (1,)), "f32")
    s.output(s.reduce("prod", xi, (1,), keep=True), "f16")
    s.output(s.apply("exp", xi), "f32")                       # an empty element-wise output next to them
    expr = G.ewf.Expression(s)
    dev = [torch.from_numpy(x).cuda()]
    big = torch.full((5, 6), 7.0, device="cuda")
    outs = [big[:, ::2], torch.full((5, 1, 3), 7.0, dtype=torch.float16, device="cuda"), torch.empty((5, 0, 3), device="cuda")]
    assert expr.output_shapes(dev) == [(5, 3), (5, 1, 3), (5, 0, 3)]
    expr.run(dev, outs, (), None, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = oracle.evaluate(s, [x])
    assert np.array_equal(outs[0].cpu().numpy(), want[0]) and np.all(want[0] == 0)
    assert np.array_equal(outs[1].cpu().numpy(), want[1]) and np.all(want[1] == 1)
    assert torch.all(big[:, 1::2] == 7.0)                     # the strided fill stayed inside its view


def test_values_computed_from_reductions_over_an_empty_axis(oracle, G):
    # log(1 + sum) + b and prod * b over an empty middle axis, next to a plain sum and an empty output
    rng = np.random.default_rng(17)
    x = np.zeros((5, 0, 3), np.float32)
    b = rng.standard_normal((5, 1, 3)).astype(np.float32)
    s = GraphSpec(3)
    xi = s.input("f32", (False,) * 3); bi = s.input("f32", (False, True, False))
    total = s.reduce("sum", xi, (1,), keep=True)
    s.output(s.add(s.apply("log1p", total), bi), "f32")
    s.output(s.mul(s.reduce("prod", s.mul(xi, bi), (1,)), s.const(3.0)), "f32")
    s.output(s.reduce("sum", xi, (1,)), "f32")
    s.output(s.mul(xi, bi), "f32")
    print("[case] expressions of reductions over an empty axis", flush=True)
    expr, got = run_spec(G, s, [x, b])
    assert expr.info()["kernel_class"] == "multi"
    want = oracle.evaluate(s, [x, b])
    assert [g_.shape for g_ in got] == [(5, 1, 3), (5, 3), (5, 3), (5, 0, 3)]
    for g_, w_ in zip(got, want):
        assert np.array_equal(g_, w_)
    assert np.array_equal(got[0], b) and np.all(got[1] == 3.0)
    # the same through the entry point that uses the library's own workspace
    import torch
    dev = [torch.from_numpy(x).cuda(), torch.from_numpy(b).cuda()]
    outs = G.h.alloc_outputs(expr, s, dev, fill=7)
    expr.plan(dev, outs)
    expr.run_static(dev, outs, (), torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    for o_, w_ in zip(outs, want):
        assert np.array_equal(o_.cpu().numpy(), w_)


def test_every_reduction_kind_row_and_split(oracle, G):
    rng = np.random.default_rng(18)
    for shape, axes in [((200, 333), (1,)), ((3, 40000), (1,)), ((6, 5, 2000), (0, 2))]:
        nd = len(shape)
        X = rng.uniform(0.9, 1.1, shape).astype(np.float32)
        I = rng.integers(-1000, 1000, shape).astype(np.int32)
        s = GraphSpec(nd)
        x = s.input("f32", (False,) * nd); i = s.input("i32", (False,) * nd)
        for red in ("sum", "max", "min"):
            s.output(s.reduce(red, x, axes), "f32")
            s.output(s.reduce(red, i, axes), "i32")
        if shape[0] != 3:
            s.output(s.reduce("prod", s.apply("sqrt", s.apply("sqrt", x)), axes), "f32")
        if len(axes) == 1:
            s.output(s.reduce("argmax", x, axes), "i32")
            s.output(s.reduce("argmax", i, axes), "i32")
        print(f"[case] reductions {shape} axes {axes}", flush=True)
        expr, got = run_spec(G, s, [X, I])
        want = oracle.evaluate(s, [X, I], nthreads=4)
        for k, ((v, st), g_, w_) in enumerate(zip(s.outputs, got, want)):
            if st == "i32":
                G.h.compare(f"{shape}.out{k}", g_, w_, 0, 0)
            else:
                G.h.compare(f"{shape}.out{k}", g_, w_, 1e-5, 1e-6)


def test_column_reductions(oracle, G):
    # reduced axes that are not the fastest-varying ones: the lanes run along the kept axis
    rng = np.random.default_rng(183)
    cases = [((1000, 64), (0,)), ((37, 5, 48), (0,)), ((37, 5, 48), (1,)), ((6, 50, 7, 32), (0, 2)), ((300, 3), (0,)),
             ((5, 4096), (0,)), ((70000, 8), (0,)), ((3, 9, 1000), (0, 1)), ((129, 260), (0,))]
    for shape, axes in cases:
        nd = len(shape)
        X = rng.uniform(0.9, 1.1, shape).astype(np.float32)
        I = rng.integers(-1000, 1000, shape).astype(np.int32)
        s = GraphSpec(nd)
        x = s.input("f32", (False,) * nd); i = s.input("i32", (False,) * nd)
        for red in ("sum", "max", "min"):
            s.output(s.reduce(red, x, axes), "f32")
            s.output(s.reduce(red, i, axes), "i32")
        s.output(s.reduce("sum", s.apply("tanh", s.mul(x, x)), axes), "f32")
        if len(axes) == 1:
            s.output(s.reduce("argmax", x, axes), "i32")
            s.output(s.reduce("argmax", i, axes), "i32")
        s.output(s.apply("exp", x), "f32")                    # an element-wise output in the same pass
        print(f"[case] column reductions {shape} axes {axes}", flush=True)
        expr, got = run_spec(G, s, [X, I])
        assert expr.info()["kernel_class"] == "col", expr.info()
        want = oracle.evaluate(s, [X, I], nthreads=4)
        for k, ((v, st), g_, w_) in enumerate(zip(s.outputs, got, want)):
            if st == "i32":
                G.h.compare(f"{shape}.out{k}", g_, w_, 0, 0)
            elif k == len(s.outputs) - 1:
                G.h.compare(f"{shape}.exp", g_, w_, 2e-6, 1e-6)
            else:
                G.h.compare(f"{shape}.out{k}", g_, w_, 1e-5, 1e-6)


def test_column_reduction_special_cases(oracle, G):
    rng = np.random.default_rng(184)
    # integer-valued float sums are exact whatever the order; ties, NaN and -inf columns for arg-max
    X = rng.integers(-20, 20, (5000, 40)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    s.output(s.reduce("sum", xi, (0,)), "f32")
    s.output(s.reduce("argmax", xi, (0,)), "i32")
    s.output(s.reduce("max", xi, (0,)), "f32")
    X[:, 1] = -np.inf
    X[7, 2] = np.nan; X[99, 2] = np.nan
    X[:, 3] = 2.0
    expr, got = run_spec(G, s, [X])
    assert expr.info()["kernel_class"] == "col"
    want = oracle.evaluate(s, [X], nthreads=4)
    assert np.array_equal(got[0], want[0], equal_nan=True)
    assert np.array_equal(got[1], want[1]) and got[1][1] == 0 and got[1][2] == 7 and got[1][3] == 0
    assert np.array_equal(got[2], want[2], equal_nan=True)
    # float16 storage, a broadcast operand and a transposed view whose reduced axis is the slow one
    A = rng.uniform(-1, 1, (64, 300)).astype(np.float16)
    Bv = rng.uniform(0.5, 1.5, (1, 300)).astype(np.float16)
    s = GraphSpec(2)
    a = s.input("f16", (False, False)); b = s.input("f16", (True, False))
    s.output(s.reduce("sum", s.mul(a, b), (0,)), "f32")
    s.output(s.mul(a, b), "f16")
    expr, got = run_spec(G, s, [A, Bv])
    assert expr.info()["kernel_class"] == "col"
    want = oracle.evaluate(s, [A, Bv])
    G.h.compare("f16 colsum", got[0], want[0], 1e-5, 1e-6)
    assert np.array_equal(got[1], want[1])
    T = rng.standard_normal((96, 200)).astype(np.float32).T           # logical [200, 96], strides (1, 200)
    s = GraphSpec(2)
    s.output(s.reduce("sum", s.apply("abs", s.input("f32", (False, False))), (1,)), "f32")
    expr, got = run_spec(G, s, [T])
    assert expr.info()["kernel_class"] == "col", expr.info()
    G.h.compare("transposed", got[0], oracle.evaluate(s, [T])[0], 1e-5, 1e-6)


def test_plans_in_several_passes(oracle, G):
    # structures no single kernel class covers: reductions are materialised stage by stage
    rng = np.random.default_rng(186)
    # batch normalisation over axis 0: mean, then variance of the centred values, then the normalised tensor
    x = rng.standard_normal((300, 70)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    inv_n = s.const(1.0 / 300)
    mean = s.mul(s.reduce("sum", xi, (0,), keep=True), inv_n)
    cen = s.sub(xi, mean)
    var = s.mul(s.reduce("sum", s.apply("sqr", cen), (0,), keep=True), inv_n)
    s.output(s.div(cen, s.apply("sqrt", s.add(var, s.const(1e-5)))), "f32")
    s.output(mean, "f32"); s.output(var, "f32")
    print("[case] batch normalisation in stages", flush=True)
    expr, got = run_spec(G, s, [x])
    # mean and sum of squared deviations in one sweep (single-pass accumulator), the normalised tensor in a second
    assert expr.info()["kernel_class"] == "multi" and expr.info()["grid_blocks"] == 2
    assert "sum of squared deviations" in expr.source(0)
    want = oracle.evaluate(s, [x])
    G.h.compare("normalised", got[0], want[0], 1e-5, 1e-6)
    G.h.compare("mean", got[1], want[1], 1e-5, 1e-6); G.h.compare("var", got[2], want[2], 1e-5, 1e-6)
    # reductions over unrelated axis sets, an arg-max among them, dropped axes in the outputs
    y = rng.standard_normal((40, 50, 12)).astype(np.float32)
    s = GraphSpec(3)
    yi = s.input("f32", (False,) * 3)
    s.output(s.reduce("sum", yi, (0,)), "f32")
    s.output(s.reduce("max", yi, (1, 2)), "f32")
    s.output(s.reduce("argmax", yi, (1,)), "i32")
    s.output(s.apply("tanh", yi), "f32")
    print("[case] three axis sets", flush=True)
    expr, got = run_spec(G, s, [y])
    assert expr.info()["kernel_class"] == "multi"
    want = oracle.evaluate(s, [y])
    assert [g_.shape for g_ in got] == [(50, 12), (40,), (40, 12), (40, 50, 12)]
    G.h.compare("sum0", got[0], want[0], 1e-5, 1e-6); G.h.compare("max12", got[1], want[1], 0, 0)
    G.h.compare("argmax1", got[2], want[2], 0, 0); G.h.compare("tanh", got[3], want[3], 2e-6, 1e-6)
    # a per-row value combined with a reduction over the rows (loss minus mean loss), and a softmax along an outer axis
    z = (rng.standard_normal((64, 33)) * 2).astype(np.float32)
    s = GraphSpec(2)
    zi = s.input("f32", (False, False))
    m = s.reduce("max", zi, (0,), keep=True)
    e = s.apply("exp", s.sub(zi, m))
    p = s.div(e, s.reduce("sum", e, (0,), keep=True))                    # softmax down the columns
    rowsum = s.reduce("sum", p, (1,), keep=True)
    s.output(p, "f32")
    s.output(s.sub(rowsum, s.mul(s.reduce("sum", rowsum, (0,), keep=True), s.const(1.0 / 64))), "f32")
    print("[case] column softmax and centred row sums", flush=True)
    expr, got = run_spec(G, s, [z])
    assert expr.info()["kernel_class"] == "multi"
    want = oracle.evaluate(s, [z])
    G.h.compare("p", got[0], want[0], 1e-5, 1e-7); G.h.compare("centred", got[1], want[1], 1e-5, 1e-6)


def _moments_spec(ndim, axes, n, storage="f32", divide=False):
    """mean, variance of the centred values (biased), and the normalised tensor over `axes`."""
    s = GraphSpec(ndim)
    xi = s.input(storage, (False,) * ndim)
    total = s.reduce("sum", xi, axes, keep=True)
    mean = s.div(total, s.const(float(n))) if divide else s.mul(total, s.const(1.0 / n))
    cen = s.sub(xi, mean)
    var = s.mul(s.reduce("sum", s.mul(cen, cen), axes, keep=True), s.const(1.0 / n))
    s.output(mean, "f32"); s.output(var, "f32")
    s.output(s.mul(cen, s.apply("recip", s.apply("sqrt", s.add(var, s.const(1e-5))))), storage)
    return s


@pytest.mark.parametrize("shape,axes,storage,offset,first", [
    ((4099, 300), (0,), "f32", 0.0, "col"),             # batch normalisation of a matrix
    ((4099, 300), (0,), "f32", 1000.0, "col"),          # a mean a thousand deviations away from zero
    ((70001, 24), (0,), "f16", 3.0, "col"),
    ((33, 20, 17, 19), (0, 2, 3), "f32", -50.0, "tile_reduce"),   # per-channel statistics of feature maps
    ((6, 150001), (1,), "f32", 10.0, "tile_reduce"),    # rows too long for the registers of a workgroup
    ((3, 5, 7), (0, 1, 2), "f32", 2.0, None),
])
def test_mean_and_variance_in_one_sweep(shape, axes, storage, offset, first, oracle, G):
    """mean -> variance of the centred values is a chain of two reductions; outside the row class
    (where the data waits in registers) the planner makes it one level with the single-pass
    (count, mean, sum of squared deviations) accumulator, so the tensor is read twice, not three
    times.  Against the oracle's two-pass evaluation in float64."""
    rng = np.random.default_rng(300 + len(shape) + int(offset))
    x = (rng.standard_normal(shape) * 1.5 + offset).astype(np.float16 if storage == "f16" else np.float32)
    n = int(np.prod([shape[d] for d in axes]))
    for divide in (False, True):
        s = _moments_spec(len(shape), axes, n, storage, divide)
        print(f"[case] moments {shape} over {axes} {storage} offset {offset} divide {divide}", flush=True)
        expr, got = run_spec(G, s, [x])
        info = expr.info()
        if first is not None:
            assert info["kernel_class"] == "multi" and info["grid_blocks"] == 2, info
            assert expr.info(0)["kernel_class"] == first and "sum of squared deviations" in expr.source(0)
        want = oracle.evaluate(s, [x], nthreads=4)
        x64 = x.astype(np.float64)
        G.h.compare("mean", got[0], want[0], 1e-5, 1e-6, scale=np.abs(x64).sum(axes, keepdims=True) / n)
        G.h.compare("var", got[1], want[1], 1e-5, 1e-6)
        # x - mean cancels: the rounding of x and of the mean, relative to the deviation, is what the
        # float32 result can know, so the bar is relative to (|x| + |mean|) / deviation
        spread = np.sqrt(x64.var(axes, keepdims=True) + 1e-5)
        if storage == "f32":
            G.h.compare("normalised", got[2], want[2], 1e-5, 1e-6, scale=(np.abs(x64) + np.abs(x64.mean(axes, keepdims=True))) / spread)
        else:
            G.h.compare("normalised", got[2], want[2], 2e-3, 1e-3)
    # a divisor that is not the number of elements is not a mean: the chain stays as described
    # (checked where the data is not far from zero: as described in float32, the subtraction of a
    # rounded mean of about 1000 alone costs more than the bar allows)
    if abs(offset) > 10:
        return
    s = _moments_spec(len(shape), axes, n + 1, storage)
    expr, got = run_spec(G, s, [x])
    stages = expr.info()["grid_blocks"] if expr.info()["kernel_class"] == "multi" else 0
    assert "sum of squared deviations" not in expr.source() + "".join(expr.source(k) for k in range(stages))
    want = oracle.evaluate(s, [x], nthreads=4)
    G.h.compare("var with another divisor", got[1], want[1], 1e-5, 1e-6)


def test_gradient_of_a_product_reduction(oracle, G):
    # the library differentiates prod over an axis (zeros handled: one zero in a row, several in another)
    rng = np.random.default_rng(187)
    x = (rng.uniform(0.9, 1.1, (37, 130)) * np.where(rng.random((37, 130)) < 0.3, -1, 1)).astype(np.float32)
    x[5, 17] = 0.0; x[9, 3] = 0.0; x[9, 129] = 0.0
    c = rng.standard_normal((37, 1)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); ci = s.input("f32", (False, True))
    (gx,) = s.grad([s.reduce("prod", xi, (1,), keep=True)], [ci], [xi])
    s.output(gx, "f32")
    print("[case] gradient of a row product", flush=True)
    expr, got = run_spec(G, s, [x, c])
    want = oracle.evaluate(G.ewf.export_spec(s), [x, c])
    assert np.count_nonzero(want[0][9]) == 0 and np.count_nonzero(want[0][5]) == 1
    G.h.compare("dprod", got[0], want[0], 1e-5, 1e-6)


def test_gradient_through_a_sum_reaches_operands_constant_along_it(oracle, G):
    # y = sum over rows of (x * w + b): b is used once per row, so db = rows * ybar; dx has x's shape
    # although nothing it is computed from varies along the rows
    rng = np.random.default_rng(188)
    R, C = 301, 1030
    x = rng.standard_normal((R, C)).astype(np.float32)
    w = rng.uniform(0.5, 1.5, (1, C)).astype(np.float32); b = rng.standard_normal((1, C)).astype(np.float32)
    ybar = rng.standard_normal((1, C)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); wi = s.input("f32", (True, False)); bi = s.input("f32", (True, False))
    yb = s.input("f32", (True, False))
    y = s.reduce("sum", s.add(s.mul(xi, wi), bi), (0,), keep=True)
    for g_ in s.grad([y], [yb], [xi, wi, bi]):
        s.output(g_, "f32")
    print("[case] gradient of a column sum with respect to row operands", flush=True)
    expr, got = run_spec(G, s, [x, w, b, ybar])
    want = oracle.evaluate(G.ewf.export_spec(s), [x, w, b, ybar])
    assert got[0].shape == (R, C) and got[1].shape == (1, C) and got[2].shape == (1, C)
    assert np.array_equal(want[0], np.broadcast_to(ybar * w, (R, C))) and np.array_equal(want[2], np.float32(R) * ybar)
    G.h.compare("dx", got[0], want[0], 2e-6, 1e-6)
    G.h.compare("dw", got[1], want[1], 1e-5, 1e-6, scale=np.abs(ybar.astype(np.float64) * x).sum(0, keepdims=True))   # terms of either sign
    G.h.compare("db", got[2], want[2], 1e-5, 1e-6)


@pytest.mark.parametrize("shape,ops", [((64, 3000), ("tanh", "sigmoid")), ((64, 7), ("sigmoid", "exp")), ((5, 3000), ("tanh", "log"))])
def test_gradient_of_a_maximum_finds_its_element_in_every_kernel(shape, ops, oracle, G):
    # The cotangent of max goes to the elements equal to it.  A plan in two kernels folds the maximum
    # in the first and compares every element with it in the second: both must evaluate the
    # expression with the same routines, to the last bit, or the comparison finds nothing.
    rng = np.random.default_rng(2049)
    R, C = shape
    a = rng.uniform(0.5, 1.5, (R, C)).astype(np.float32); b = rng.uniform(0.5, 1.5, (1, C)).astype(np.float32)
    cot = rng.standard_normal((R, 1)).astype(np.float32)
    s = GraphSpec(2)
    ai = s.input("f32", (False, False)); bi = s.input("f32", (True, False)); ci = s.input("f32", (False, True))
    v = s.add(s.apply(ops[0], s.mul(ai, bi)), s.apply(ops[1], ai))
    red = s.reduce("max", s.mul(v, s.const(0.5)), (1,), keep=True)
    ga, gb = s.grad([red], [ci], [ai, bi])
    s.output(ga, "f32"); s.output(gb, "f32")
    print(f"[case] gradient of a row maximum {shape} {ops}", flush=True)
    for opts in ({}, {"split_rows": 1}, {"tile_elems": 1024}):
        try:
            expr, got = run_spec(G, s, [a, b, cot], **opts)
        except G.ewf.EwfError as e:
            assert e.status == G.ewf.EUNSUPPORTED
            continue
        want = oracle.evaluate(G.ewf.export_spec(s), [a, b, cot])
        hit = want[0] != 0                                  # one element per row (no ties in this data)
        assert hit.sum() == R and (got[0] != 0).sum() == R, (opts, expr.info()["kernel_class"], int((got[0] != 0).sum()))
        assert np.array_equal(got[0] != 0, hit)
        G.h.compare("da", got[0], want[0], 1e-5, 1e-6)
        G.h.compare("db", got[1], want[1], 1e-5, 1e-6)          # a column sums the few rows whose maximum lies in it


def test_argmax_ties_take_the_first_index(oracle, G):
    x = np.zeros((70, 5000), np.float32)
    x[:, 4000] = 3.0; x[:, 123] = 3.0; x[5, 7] = 3.0
    x[9, :] = -np.inf
    s = GraphSpec(2)
    s.output(s.reduce("argmax", s.input("f32", (False, False)), (1,)), "i32")
    for opts in ({}, {"block_threads": 64}, {"block_threads": 1024}):
        _, (got,) = run_spec(G, s, [x], **opts)
        want = oracle.evaluate(s, [x])[0]
        assert np.array_equal(got, want)
        assert got[0] == 123 and got[5] == 7 and got[9] == 0


def test_max_shares_the_argmax_accumulator(oracle, G):
    # max and arg-max of one argument share an accumulator; NaN wins both (first NaN), a row of
    # -inf gives index 0, equal maxima the first index -- in the row class and the split class
    rng = np.random.default_rng(181)
    for shape in [(600, 700), (3, 50000)]:
        x = rng.standard_normal(shape).astype(np.float32)
        x[0, :] = -np.inf
        x[1, 5] = np.nan; x[1, 400] = np.nan; x[1, 17] = 9.0
        x[2, 3::64] = 7.0
        if shape[0] > 3:
            x[3, :] = -np.inf; x[3, 699] = -1e30
            x[4, :] = 2.5
        s = GraphSpec(2)
        xi = s.input("f32", (False, False))
        s.output(s.reduce("max", xi, (1,)), "f32")
        s.output(s.reduce("argmax", xi, (1,)), "i32")
        s.output(s.reduce("sum", s.apply("abs", s.apply("tanh", xi)), (1,)), "f32")
        print(f"[case] shared max/argmax {shape}", flush=True)
        expr, got = run_spec(G, s, [x])
        want = oracle.evaluate(s, [x], nthreads=4)
        assert np.array_equal(got[0], want[0], equal_nan=True), expr.info()
        assert np.array_equal(got[1], want[1]), expr.info()
        assert got[1][0] == 0 and got[1][1] == 5 and got[1][2] == 3
        G.h.compare("sum", got[2], want[2], 1e-5, 1e-6)


def test_one_hot_sum_is_read_as_a_gather(oracle, G):
    # sum_j where(iota_j == t, x_j, 0) is one element of x: the row class reads it directly.
    # Out-of-range indices give 0, a NaN elsewhere in the row does not leak, -0 becomes +0.
    rng = np.random.default_rng(182)
    rows, cols = 700, 333
    x = rng.standard_normal((rows, cols)).astype(np.float32)
    t = rng.integers(0, cols, (rows, 1)).astype(np.int32)
    t[0, 0] = -1; t[1, 0] = cols; t[2, 0] = 2**31 - 1; t[3, 0] = 0; t[4, 0] = cols - 1
    x[5, :] = np.nan; x[5, 7] = 1.25; t[5, 0] = 7
    x[6, 9] = -0.0; t[6, 0] = 9
    for storage, tol in (("f32", 0.0), ("f16", 0.0)):
        xs = x.astype(np.float16) if storage == "f16" else x
        s = GraphSpec(2)
        xi = s.input(storage, (False, False)); ti = s.input("i32", (False, True))
        hit = s.apply("eq", ti, s.iota(1)) if storage == "f16" else s.apply("eq", s.iota(1), ti)
        s.output(s.reduce("sum", s.apply("where", hit, xi, s.const(0.0)), (1,)), "f32")
        s.output(s.reduce("sum", s.apply("abs", xi), (1,)), "f32")
        print(f"[case] one-hot sum as gather, {storage}", flush=True)
        expr, got = run_spec(G, s, [xs, t])
        assert expr.info()["kernel_class"] == "row" and "(idx_t)(in_ ? t_ : 0)" in expr.source()
        want = oracle.evaluate(s, [xs, t], nthreads=4)
        assert np.array_equal(got[0], want[0]) and not np.signbit(got[0][6])
        assert got[0][0] == 0 and got[0][1] == 0 and got[0][2] == 0 and got[0][5] == 1.25
        G.h.compare("abs-sum", got[1], want[1], 1e-5, 1e-6)


def test_softmax_probabilities_row_class(oracle, G):
    rng = np.random.default_rng(19)
    for rows, cols in [(33, 1000), (5, 9000), (700, 24)]:
        x = (rng.standard_normal((rows, cols)) * 3).astype(np.float32)
        s = GraphSpec(2)
        xi = s.input("f32", (False, False))
        e = s.apply("exp", s.sub(xi, s.reduce("max", xi, (1,))))
        p = s.div(e, s.reduce("sum", e, (1,)))
        s.output(p, "f32")
        s.output(s.reduce("sum", p, (1,)), "f32")          # third chained level: rows sum to one
        print(f"[case] softmax {rows}x{cols}", flush=True)
        expr, (gp, gs) = run_spec(G, s, [x])
        assert expr.info()["kernel_class"] == "row"
        wp, wsum = oracle.evaluate(s, [x], nthreads=4)
        G.h.compare("p", gp, wp, 1e-5, 1e-7)
        G.h.compare("rowsum", gs, wsum, 1e-5, 1e-6)
        assert np.allclose(gs, 1.0, atol=1e-5)


def test_streaming_rows_longer_than_registers(oracle, G):
    # rows too long to stay in registers are re-read level by level
    rng = np.random.default_rng(20)
    x = (rng.standard_normal((4, 70000)) * 2).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    m = s.reduce("max", xi, (1,))
    S = s.reduce("sum", s.apply("exp", s.sub(xi, m)), (1,))
    s.output(s.add(m, s.apply("log", S)), "f32")
    want = oracle.evaluate(s, [x], nthreads=4)[0]
    expr, (got,) = run_spec(G, s, [x], split_rows=2, no_rewrite=1)
    assert expr.info()["kernel_class"] == "row"
    G.h.compare("lse", got, want, 1e-5, 1e-6)
    # left to itself the library makes the chain one rescaled level and splits the rows over
    # workgroups; a second, tiny pass computes the result from the level's pair
    expr, (got,) = run_spec(G, s, [x])
    assert expr.info()["kernel_class"] == "multi" and expr.info(0)["kernel_class"] == "tile_reduce", expr.info()
    assert "* w_ + 1.0f" in expr.source(0)
    G.h.compare("lse_split", got, want, 1e-5, 1e-6)


# ------------------------------------------------------------------ random graphs

SAFE_UN = ["neg", "abs", "exp", "log1p", "sqrt", "tanh", "sigmoid", "sqr", "recip", "expm1", "log"]


def random_case(seed):
    rng = np.random.default_rng(7000 + seed)
    ndim = int(rng.integers(1, 5))
    full = [int(rng.choice([1, 2, 3, 5, 8, 13, 32, 40])) for _ in range(ndim)]
    if rng.integers(0, 2):
        full[-1] = int(rng.choice([4, 16, 64, 100, 256]))
    s = GraphSpec(ndim)
    inputs, vals = [], []
    for k in range(int(rng.integers(1, 4))):
        bc = tuple(bool(rng.integers(0, 4) == 0) and k > 0 for _ in range(ndim))
        shp = [1 if b else e for b, e in zip(bc, full)]
        style = int(rng.integers(0, 3))
        if style == 0:
            view = rng.uniform(0.2, 2.0, shp).astype(np.float32)
        elif style == 1:                                  # slice of a larger buffer
            big = rng.uniform(0.2, 2.0, [e + 3 for e in shp]).astype(np.float32)
            view = big[tuple(slice(1, 1 + e) for e in shp)]
        else:                                             # permuted and strided
            perm = rng.permutation(ndim)
            big = rng.uniform(0.2, 2.0, [2 * shp[p] + 1 for p in perm]).astype(np.float32)
            view = big.transpose(np.argsort(perm))[tuple(slice(1, 1 + 2 * e, 2) for e in shp)]
        inputs.append(view)
        vals.append(s.input("f32", bc))
    vals.append(s.scalar("f32"))
    reduce_axes = None
    if rng.integers(0, 2):
        # trailing axes of a contiguous operand, or (every other case) any subset of the axes
        k = int(rng.integers(1, ndim + 1))
        reduce_axes = tuple(range(ndim - k, ndim))
        if seed % 2:
            reduce_axes = tuple(sorted(rng.choice(ndim, size=int(rng.integers(1, ndim + 1)), replace=False).tolist()))
        inputs[0] = np.ascontiguousarray(inputs[0])
    for _ in range(int(rng.integers(2, 8))):
        r = rng.integers(0, 10)
        a = vals[int(rng.integers(len(vals)))]
        if r < 4:
            op = SAFE_UN[int(rng.integers(len(SAFE_UN)))]
            if op in ("log", "recip"):
                v = s.apply(op, s.add(s.apply("abs", a), s.const(0.5)))
            elif op in ("sqrt", "log1p"):
                v = s.apply(op, s.apply("abs", a))
            else:
                v = s.apply(op, a)
        elif r < 8:
            op = ["add", "mul", "max", "min", "sub"][int(rng.integers(5))]
            v = s.apply(op, a, vals[int(rng.integers(len(vals)))])
        else:
            b, c = (vals[int(rng.integers(len(vals)))] for _ in range(2))
            v = s.apply("where", s.apply("gt", a, b), c, a)
        v = s.apply("tanh", v) if rng.integers(0, 3) == 0 else v
        vals.append(v)
    s.output(vals[-1], "f32")
    kinds, aux_outputs = ["elementwise"], []
    if reduce_axes is not None:
        x0 = vals[0]
        red = ["sum", "max", "min"][int(rng.integers(3))]
        keep = bool(seed % 3 == 2)
        term = s.apply("tanh", s.mul(x0, vals[-1]))
        r_ = s.reduce(red, term, reduce_axes, keep=keep)
        s.output(r_, "f32"); kinds.append(red)
        if keep:                                            # a value normalised by the reduction (may need several passes)
            s.output(s.sub(vals[-1], r_), "f32"); kinds.append("normalised")
        first = int(rng.integers(0, 2))                     # sometimes reduce-only
        s.outputs = s.outputs[first:]; kinds = kinds[first:]
        aux_outputs = [("sum" if red == "sum" else "max", term, reduce_axes, keep), vals[-1]]
    # what the bars of the outputs are relative to, as a description of its own for the oracle: for a
    # sum the sum of the magnitudes of its terms (for max / min the largest magnitude), and |last value|
    aux = GraphSpec(ndim); aux.nodes = list(s.nodes); aux.n_inputs = s.n_inputs; aux.n_scalars = s.n_scalars
    if aux_outputs:
        (red, term, axes, keep), last = aux_outputs
        aux.output(aux.reduce(red, aux.apply("abs", term), axes, keep=keep), "f32")
        aux.output(aux.apply("abs", last), "f32")
    return s, inputs, [float(rng.uniform(0.5, 1.5))], aux, kinds


@pytest.mark.parametrize("seed", range(60))
def test_random_graphs_and_layouts(seed, oracle, G):
    s, inputs, scal, aux, kinds = random_case(seed)
    print(f"[case] fuzz seed {seed} ndim {s.ndim} shapes {[a.shape for a in inputs]} strides "
          f"{[tuple(x // 4 for x in a.strides) for a in inputs]} outputs {len(s.outputs)}", flush=True)
    want = oracle.evaluate(s, inputs, scal)
    magnitude = [m.astype(np.float64) for m in oracle.evaluate(aux, inputs, scal)] if aux.outputs else []
    try:
        expr, got = run_spec(G, s, inputs, scal)
    except G.ewf.EwfError as e:
        if e.status == G.ewf.EUNSUPPORTED:
            pytest.skip(f"layout not covered by a kernel class: {e.message}")
        raise
    for k, (g_, w_, kind, (v, _)) in enumerate(zip(got, want, kinds, s.outputs)):
        # A chain of d rounding operations: d times the element-wise bar (every operation adds its
        # own rounding to what it received; the generator keeps arguments where no operation
        # amplifies that by more than the bar allows for).  A sum adds the bar for reductions,
        # relative to the magnitudes of its terms; a value minus a reduction is held to the
        # magnitudes of both.
        d = G.h.rounding_depth(s, v)
        if kind in ("elementwise", "max", "min"):
            G.h.compare(f"seed{seed}.out{k}", g_, w_, 2e-6 * d, 1e-6 * d)
        elif kind == "sum":
            G.h.compare(f"seed{seed}.out{k}", g_, w_, 1e-5 + 2e-6 * d, 1e-6 * d, scale=magnitude[0])
        else:
            G.h.compare(f"seed{seed}.out{k}", g_, w_, 1e-5 + 2e-6 * d, 1e-6 * d, scale=magnitude[0] + magnitude[1])


# ------------------------------------------------------------------ softmax chains split over workgroups

def _lse_spec(storage="f32", axis=1):
    """max, sum of exp(x - max), log-sum-exp and the softmax probabilities along `axis`."""
    s = GraphSpec(2)
    x = s.input(storage, (False, False))
    m = s.reduce("max", x, (axis,), keep=True)
    ex = s.apply("exp", s.sub(x, m))
    S = s.reduce("sum", ex, (axis,), keep=True)
    s.output(m, "f32"); s.output(S, "f32")
    s.output(s.add(m, s.apply("log", S)), "f32")
    s.output(s.div(ex, S), storage)
    return s


def test_long_rows_are_split_and_the_exp_sum_is_rescaled_online(oracle, G):
    from workloads import configs as wl
    # rows too long for the registers of a workgroup: the chain max -> sum of exp becomes one level
    w = wl.c3_softmax_xent(rows=37, vocab=150001)
    print(f"[case] {w.name} 37 x 150001", flush=True)
    expr, stats = G.h.check_workload(w, oracle)
    info = expr.info()
    assert info["kernel_class"] == "multi", info
    assert expr.info(0)["kernel_class"] == "tile_reduce" and "b2 * w_" in expr.source(0).replace("acc.", "")
    w = wl.c3_softmax_xent_backward(rows=5, vocab=70001)
    print(f"[case] {w.name} 5 x 70001", flush=True)
    expr, stats = G.h.check_workload(w, oracle)
    assert expr.info()["kernel_class"] == "multi" and expr.info()["grid_blocks"] == 2
    # few rows that would fit: one workgroup per row would leave the chip idle
    rng = np.random.default_rng(188)
    x = (rng.standard_normal((3, 40000)) * 3).astype(np.float32)
    s = _lse_spec()
    print("[case] 3 x 40000 softmax", flush=True)
    expr, got = run_spec(G, s, [x])
    assert expr.info()["kernel_class"] == "multi"
    want = oracle.evaluate(s, [x])
    for name, g_, w_ in zip(("max", "expsum", "lse", "p"), got, want):
        G.h.compare(name, g_, w_, 1e-5, 1e-9 if name == "p" else 1e-6)


@pytest.mark.parametrize("storage,axis", [("f32", 1), ("f16", 1), ("f32", 0)])
def test_split_softmax_at_small_sizes_and_special_values(storage, axis, oracle, G):
    rng = np.random.default_rng(189)
    dt = np.float32 if storage == "f32" else np.float16
    x = (rng.standard_normal((41, 1003)) * 4).astype(dt)
    inf = dt(np.inf)
    x[1, 5] = -inf; x[1, 900] = -inf                       # terms that vanish
    x[2, :] = -inf                                          # nothing but -inf: NaN as described
    x[3, 0] = -inf; x[3, 1] = 2.0                           # the first elements a thread meets are -inf
    x[4, 77] = inf                                          # inf - inf
    x[5, 500] = np.nan
    x[6, :] = 1.5                                           # every element the maximum
    x[7, :] = -3.0e38 if storage == "f32" else -60000.0     # the most negative numbers
    x[8, 1002] = 80.0 if storage == "f32" else 30.0         # the maximum arrives last: everything before is rescaled
    if axis == 0:
        x = np.ascontiguousarray(x.T)
    s = _lse_spec(storage, axis)
    print(f"[case] split softmax {storage} axis {axis}", flush=True)
    expr, got = run_spec(G, s, [x], split_rows=1)
    assert expr.info()["kernel_class"] == "multi", expr.info()
    want = oracle.evaluate(s, [x])
    tol_p = (1e-5, 1e-9) if storage == "f32" else (2e-3, 1e-3)
    assert np.array_equal(got[0], want[0], equal_nan=True)
    G.h.compare("expsum", got[1], want[1], 1e-5, 1e-6)
    G.h.compare("lse", got[2], want[2], 1e-5, 1e-6)
    G.h.compare("p", got[3], want[3], *tol_p)
    # and the same description with one workgroup per row agrees
    if axis == 1:
        expr2, got2 = run_spec(G, s, [x], split_rows=2)
        assert expr2.info()["kernel_class"] == "row"
        G.h.compare("expsum_row", got2[1], want[1], 1e-5, 1e-6)


@pytest.mark.parametrize("seed", range(12))
def test_random_softmax_chains(seed, oracle, G):
    """max -> sum of exp(. - max) chains along a random axis of random shapes, with one workgroup
    per row, split over workgroups, and whatever the library picks."""
    rng = np.random.default_rng(9000 + seed)
    ndim = int(rng.integers(2, 4))
    shape = [int(rng.choice([1, 3, 7, 33, 130, 257])) for _ in range(ndim)]
    axis = int(rng.integers(0, ndim))
    shape[axis] = int(rng.choice([5, 64, 1000, 4099]))
    storage = "f16" if seed % 4 == 3 else "f32"
    dt = np.float16 if storage == "f16" else np.float32
    x = (rng.standard_normal(shape) * 3).astype(dt)
    bshape = [1 if d == axis or rng.integers(0, 2) else e for d, e in enumerate(shape)]
    b = rng.standard_normal(bshape).astype(np.float32)
    s = GraphSpec(ndim)
    xi = s.input(storage, tuple(False for _ in shape))
    bi = s.input("f32", tuple(e == 1 and shape[d] > 1 for d, e in enumerate(bshape)))
    pre = int(rng.integers(0, 3))
    f = xi if pre == 0 else s.add(s.mul(xi, s.const(0.5)), bi) if pre == 1 else s.mul(s.apply("tanh", xi), s.const(4.0))
    keep = bool(rng.integers(0, 2))
    m = s.reduce("max", f, (axis,), keep=True)
    ex = s.apply("exp", s.sub(f, m))
    S = s.reduce("sum", ex, (axis,), keep=True)
    names = []
    if rng.integers(0, 2) or True:
        s.output(s.add(m, s.apply("log", S)), "f32"); names.append("lse")
    if rng.integers(0, 2):
        # of the input itself: a computed value would let rounding decide the index
        s.output(s.reduce("argmax", xi, (axis,), keep=keep), "i32"); names.append("argmax")
    if rng.integers(0, 2):
        s.output(s.div(ex, S), storage); names.append("p")
    if rng.integers(0, 2):
        s.output(s.div(s.reduce("sum", s.mul(ex, f), (axis,), keep=keep), s.reduce("sum", ex, (axis,), keep=keep)), "f32"); names.append("mean_f")
    mode = seed % 3
    print(f"[case] chain seed={seed} shape={shape} axis={axis} {storage} pre={pre} outputs={names} split_rows={mode}", flush=True)
    expr, got = run_spec(G, s, [x, b], split_rows=mode)
    want = oracle.evaluate(s, [x, b], nthreads=4)
    for name, g_, w_ in zip(names, got, want):
        if name == "argmax":
            G.h.compare(name, g_, w_, 0, 0)
        elif name == "p":
            G.h.compare(name, g_, w_, *((1e-5, 1e-8) if storage == "f32" else (2e-3, 1e-3)))
        else:
            G.h.compare(name, g_, w_, 1e-5, 1e-6)


def test_reductions_over_axes_far_apart_in_memory(oracle, G):
    # a kept dimension between the reduced ones and a short innermost run: the outer axes go
    # first (column kernel), the rest on the much smaller result
    rng = np.random.default_rng(191)
    x = rng.uniform(0.5, 1.5, (40, 30, 50, 36)).astype(np.float32)
    x *= np.where(rng.random(x.shape) < 0.5, -1, 1).astype(np.float32)
    for axes in ((1, 3), (0, 3), (0, 1, 3)):
        s = GraphSpec(4)
        xi = s.input("f32", (False,) * 4)
        s.output(s.reduce("sum", xi, axes), "f32"); s.output(s.reduce("max", xi, axes), "f32")
        s.output(s.reduce("min", xi, axes, keep=True), "f32")
        s.output(s.reduce("prod", s.add(s.mul(xi, s.const(0.01)), s.const(1.0)), axes), "f32")
        s.output(s.apply("sqrt", s.reduce("sum", s.apply("sqr", xi), axes)), "f32")       # a value computed from a split reduction
        print(f"[case] axes {axes}", flush=True)
        expr, got = run_spec(G, s, [x])
        assert expr.info()["kernel_class"] == "multi" and expr.info(0)["kernel_class"] == "col", expr.info()
        want = oracle.evaluate(s, [x], nthreads=4)
        assert [g_.shape for g_ in got] == [w_.shape for w_ in want]
        G.h.compare("sum", got[0], want[0], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64)).sum(axes)); G.h.compare("max", got[1], want[1], 0, 0)
        G.h.compare("min", got[2], want[2], 0, 0); G.h.compare("prod", got[3], want[3], G.h.product_rtol(x.size // want[3].size), 1e-6)
        G.h.compare("norm", got[4], want[4], 1e-5, 1e-6)
    # a transposed view makes the same situation out of neighbouring axes
    y = rng.standard_normal((300, 8, 700)).astype(np.float32)
    s = GraphSpec(3)
    yi = s.input("f32", (False,) * 3)
    s.output(s.reduce("sum", yi, (0, 1)), "f32")
    yt = np.ascontiguousarray(y.transpose(0, 2, 1)).transpose(0, 2, 1)      # axis 1 is now the fastest in memory
    expr, got = run_spec(G, s, [yt])
    assert expr.info()["kernel_class"] == "multi"
    G.h.compare("sum01", got[0], oracle.evaluate(s, [yt])[0], 1e-5, 1e-6, scale=np.abs(y.astype(np.float64)).sum((0, 1)))


@pytest.mark.parametrize("shape,first", [((128, 96, 14, 14), "col"), ((128, 336, 14, 14), "lane"), ((24, 448, 28, 28), "lane"), ((24, 288, 36, 36), "row")])
def test_channel_statistics_of_late_layers_with_an_elementwise_output(shape, first, oracle, G):
    # bias + ReLU + per-channel sum and maximum on feature maps whose planes are short: two passes,
    # the element-wise output written by the first one (the second reads only the first's
    # small result), the inner axes first once the tensor is large and a plane is long enough
    rng = np.random.default_rng(198 + shape[1])
    n, c, hh, ww = shape
    x = rng.standard_normal(shape).astype(np.float32)
    b = rng.standard_normal((1, c, 1, 1)).astype(np.float32)
    s = GraphSpec(4)
    xi = s.input("f32", (False,) * 4); bi = s.input("f32", (True, False, True, True))
    y = s.apply("max", s.const(0.0), s.add(xi, bi))
    s.output(y, "f32")
    s.output(s.reduce("sum", y, (0, 2, 3)), "f32")
    s.output(s.reduce("max", y, (0, 2, 3), keep=True), "f32")
    print(f"[case] {shape}", flush=True)
    expr, got = run_spec(G, s, [x, b])
    info = expr.info()
    assert info["kernel_class"] == "multi" and info["grid_blocks"] == 2, info
    assert expr.info(0)["kernel_class"] == first and expr.info(0)["extent"] == (n, c, hh * ww), expr.info(0)
    assert int(np.prod(expr.info(1)["extent"])) < x.size // 8, expr.info(1)           # nothing sweeps the tensor twice
    want = oracle.evaluate(s, [x, b], nthreads=4)
    G.h.compare("y", got[0], want[0], 2e-6, 1e-6); G.h.compare("sum", got[1], want[1], 1e-5, 1e-6)
    G.h.compare("max", got[2], want[2], 0, 0)
    # written over its input, the element-wise output waits for the last pass, which still finds
    # the input intact
    torch = G.torch
    xd = torch.from_numpy(x).cuda(); bd = torch.from_numpy(b).cuda()
    expr2 = G.ewf.Expression(s)
    outs = [xd] + G.h.alloc_outputs(expr2, s, [xd, bd])[1:]
    ws = G.h.make_workspace(expr2, [xd, bd], outs)
    expr2.run([xd, bd], outs, (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert int(np.prod(expr2.info(expr2.info()["grid_blocks"] - 1)["extent"])) == x.size
    G.h.compare("y in place", xd.cpu().numpy(), want[0], 2e-6, 1e-6)
    G.h.compare("sum", outs[1].cpu().numpy(), want[1], 1e-5, 1e-6); G.h.compare("max", outs[2].cpu().numpy(), want[2], 0, 0)


# ------------------------------------------------------------------ short rows: several rows per wavefront

@pytest.mark.parametrize("cols,storage", [(4, "f32"), (8, "f32"), (12, "f32"), (32, "f32"), (10, "f32"), (24, "f16"), (64, "f16"),
                                          (100, "f32"), (256, "f32"), (200, "f16"),
                                          # lengths that allow only narrow accesses: several per lane, or a whole row per thread
                                          (49, "f32"), (9, "f32"), (130, "f32"), (255, "f32"), (25, "f16"), (130, "f16"), (511, "f16"),
                                          # ... also beyond 1024 bytes, up to 1024 accesses per row
                                          (289, "f32"), (777, "f32"), (1001, "f16")])
def test_short_rows_share_a_wavefront(cols, storage, oracle, G):
    rng = np.random.default_rng(192 + cols)
    rows = 5003
    dt = np.float32 if storage == "f32" else np.float16
    x = (rng.standard_normal((rows, cols)) * 3).astype(dt)
    t = rng.integers(-1, cols + 1, (rows, 1)).astype(np.int32)          # some targets out of range
    x[7, :] = 2.5                                                       # ties: the first index wins
    x[8, cols - 1] = np.nan
    s = GraphSpec(2)
    xi = s.input(storage, (False, False)); ti = s.input("i32", (False, True))
    m = s.reduce("max", xi, (1,), keep=True)
    ex = s.apply("exp", s.sub(xi, m))
    S = s.reduce("sum", ex, (1,), keep=True)
    xt = s.reduce("sum", s.apply("where", s.apply("eq", s.iota(1), ti), xi, s.const(0.0)), (1,), keep=True)
    loss = s.sub(s.add(m, s.apply("log", S)), xt)
    s.output(s.div(ex, S), storage)                                     # softmax probabilities
    s.output(loss, "f32")
    s.output(s.reduce("argmax", xi, (1,)), "i32")
    s.output(s.reduce("min", xi, (1,)), "f32")
    s.output(s.div(s.reduce("sum", s.apply("where", s.apply("eq", loss, loss), loss, s.const(0.0)), (0,)), s.const(float(rows))), "f32")
    print(f"[case] short rows {rows} x {cols} {storage}", flush=True)
    expr, got = run_spec(G, s, [x, t])
    itemsize = 4 if storage == "f32" else 2
    def lanes_expected(info):
        narrow = info["vec"] * itemsize < 16
        return "lane" if cols * itemsize <= 1024 or (narrow and cols // info["vec"] <= 1024) else "row"
    assert expr.info()["kernel_class"] == lanes_expected(expr.info()), expr.info()
    want = oracle.evaluate(s, [x, t], nthreads=4)
    G.h.compare("p", got[0], want[0], *((1e-5, 1e-8) if storage == "f32" else (2e-3, 1e-3)))
    G.h.compare("loss", got[1], want[1], 1e-5, 1e-6)
    assert np.array_equal(got[2], want[2]) and got[2][7] == 0
    assert np.array_equal(got[3], want[3], equal_nan=True)
    G.h.compare("mean_loss", got[4], want[4], 1e-5, 1e-6)
    # strided rows (a slice of wider rows) and a row-constant operand
    wide = (rng.standard_normal((rows, cols + 5)) * 2).astype(dt)
    view = wide[:, 2:2 + cols]
    s2 = GraphSpec(2)
    vi = s2.input(storage, (False, False)); ci = s2.input("f32", (False, True))
    s2.output(s2.reduce("sum", s2.mul(vi, ci), (1,)), "f32")
    s2.output(s2.reduce("prod", s2.add(s2.mul(vi, s2.const(0.01)), s2.const(1.0)), (1,), keep=True), "f32")
    scale = rng.standard_normal((rows, 1)).astype(np.float32)
    expr, got = run_spec(G, s2, [view, scale])
    # the slice is not aligned for wide accesses: single elements, several of them per lane
    assert expr.info()["vec"] == 1 and expr.info()["kernel_class"] == lanes_expected(expr.info())
    want = oracle.evaluate(s2, [view, scale], nthreads=4)
    # (terms of either sign: the bar is relative to the sum of their magnitudes)
    G.h.compare("wsum", got[0], want[0], 1e-5, 1e-6, scale=np.abs(view.astype(np.float64) * scale).sum(1))
    G.h.compare("prod", got[1], want[1], 1e-5, 1e-6)


@pytest.mark.parametrize("shape,axis", [((5001, 4, 8), 1), ((3000, 3, 12), 1), ((777, 2, 5, 6), 1), ((40000, 2, 2), 1), ((9, 1100, 5, 4), 2)])
def test_short_middle_axis_with_few_columns(shape, axis, oracle, G):
    # a short reduced axis in the middle and a tiny kept innermost axis: the lanes left over take
    # neighbouring indices of the next kept dimension
    rng = np.random.default_rng(193 + len(shape))
    x = (rng.standard_normal(shape) * 2).astype(np.float32)
    nd = len(shape)
    s = GraphSpec(nd)
    xi = s.input("f32", (False,) * nd)
    s.output(s.reduce("sum", xi, (axis,)), "f32")
    s.output(s.reduce("max", xi, (axis,), keep=True), "f32")
    s.output(s.reduce("argmax", xi, (axis,)), "i32")
    s.output(s.apply("tanh", xi), "f32")                               # an element-wise output in the same pass
    print(f"[case] {shape} axis {axis}", flush=True)
    expr, got = run_spec(G, s, [x])
    assert expr.info()["kernel_class"] == "col", expr.info()
    assert expr.info()["grid_blocks"] < int(np.prod(shape[:axis])) // 4       # many outer indices per workgroup
    want = oracle.evaluate(s, [x], nthreads=4)
    G.h.compare("sum", got[0], want[0], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64)).sum(axis)); G.h.compare("max", got[1], want[1], 0, 0)
    G.h.compare("argmax", got[2], want[2], 0, 0); G.h.compare("tanh", got[3], want[3], 2e-6, 1e-6)


@pytest.mark.parametrize("storage", ["f32", "f16"])
@pytest.mark.parametrize("shape,axis", [((70001, 4, 8), 1), ((50001, 2, 16), 1), ((20011, 8, 8), 1), ((9001, 16, 16), 1), ((3, 30001, 3, 24), 2)])
def test_short_middle_axis_at_streaming_size(shape, axis, storage, oracle, G):
    # the same layout past the size where a thread keeps several loads in flight: threads with few
    # rows take several outer indices (a ragged count of them here), and the finishing threads
    # write whole vectors of columns
    rng = np.random.default_rng(197 + len(shape) + shape[-1])
    x = (rng.standard_normal(shape) * 2).astype(np.float16 if storage == "f16" else np.float32)
    nd = len(shape)
    s = GraphSpec(nd)
    xi = s.input(storage, (False,) * nd)
    s.output(s.reduce("sum", xi, (axis,)), "f32")
    s.output(s.reduce("max", xi, (axis,), keep=True), storage)
    s.output(s.reduce("argmax", xi, (axis,)), "i32")
    print(f"[case] {shape} axis {axis} {storage}", flush=True)
    expr, got = run_spec(G, s, [x])
    info = expr.info()
    assert info["kernel_class"] == "col" and info["rank"] == 3 and info["tile"][0] > 1, info
    assert "yg_out0" in expr.source() and "ewf_finish" not in expr.source()
    want = oracle.evaluate(s, [x], nthreads=4)
    G.h.compare("sum", got[0], want[0], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64)).sum(axis)); G.h.compare("max", got[1], want[1], 0, 0)
    G.h.compare("argmax", got[2], want[2], 0, 0)
    # with an element-wise output and an output computed from the sums in the same pass
    s2 = GraphSpec(nd)
    xi = s2.input(storage, (False,) * nd)
    s2.output(s2.apply("tanh", xi), storage)
    s2.output(s2.apply("sqrt", s2.reduce("sum", s2.mul(xi, xi), (axis,))), "f32")
    expr, got = run_spec(G, s2, [x])
    assert expr.info()["kernel_class"] == "col", expr.info()
    want = oracle.evaluate(s2, [x], nthreads=4)
    tol = (2e-3, 1e-3) if storage == "f16" else (2e-6, 1e-6)
    G.h.compare("tanh", got[0], want[0], *tol); G.h.compare("norm", got[1], want[1], 1e-5, 1e-6)


@pytest.mark.parametrize("shape,axes", [((6, 5001, 7, 24), (0, 2)), ((3, 40, 3001, 4, 8), (0, 1, 3)), ((5, 70001, 2, 16), (0, 2))])
def test_short_middle_axis_among_several_reduced_axes(shape, axes, oracle, G):
    # outer-index lanes when further reduced axes lie outside: their indices become slots of
    # partial results that the second kernel folds
    rng = np.random.default_rng(199 + len(shape))
    x = (rng.standard_normal(shape) * 2 + 3).astype(np.float32)        # (sums well away from zero)
    nd = len(shape)
    s = GraphSpec(nd)
    xi = s.input("f32", (False,) * nd)
    s.output(s.reduce("sum", xi, axes), "f32")
    s.output(s.reduce("max", s.apply("abs", xi), axes, keep=True), "f32")
    print(f"[case] {shape} axes {axes}", flush=True)
    expr, got = run_spec(G, s, [x])
    info = expr.info()
    assert info["kernel_class"] == "col" and "ewf_finish" in expr.source(), info
    kept = [d for d in range(info["rank"] - 1) if not info["reduced"][d]]
    assert info["tile"][kept[-1]] > 1, info                                  # several outer indices per workgroup
    want = oracle.evaluate(s, [x], nthreads=4)
    G.h.compare("sum", got[0], want[0], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64)).sum(axes)); G.h.compare("max", got[1], want[1], 0, 0)


def test_rank_zero_and_rank_eight(oracle, G):
    # the smallest and the largest rank the library accepts
    s = GraphSpec(0)
    a = s.input("f32", ()); b = s.input("f32", ())
    s.output(s.apply("tanh", s.add(a, b)), "f32")
    expr, got = run_spec(G, s, [np.array(0.25, np.float32), np.array(-1.5, np.float32)])
    G.h.compare("scalar", got[0], oracle.evaluate(s, [np.array(0.25, np.float32), np.array(-1.5, np.float32)])[0], 2e-6, 1e-6)
    rng = np.random.default_rng(194)
    shape = (2, 3, 4, 5, 2, 3, 4, 5)
    x = rng.standard_normal(shape[::-1]).astype(np.float32).transpose(7, 6, 5, 4, 3, 2, 1, 0)     # nothing merges
    y = rng.standard_normal((1, 3, 1, 5, 1, 3, 1, 5)).astype(np.float32)
    s = GraphSpec(8)
    xi = s.input("f32", (False,) * 8); yi = s.input("f32", (True, False) * 4)
    v = s.mul(xi, yi)
    s.output(s.apply("exp", v), "f32")
    s.output(s.reduce("sum", v, (1, 3, 5, 7)), "f32")
    s.output(s.reduce("max", v, (0, 2), keep=True), "f32")
    s.output(s.reduce("argmax", xi, (7,)), "i32")
    print("[case] rank 8", flush=True)
    expr, got = run_spec(G, s, [x, y])
    want = oracle.evaluate(s, [x, y])
    assert [g_.shape for g_ in got] == [w_.shape for w_ in want] == [shape, (2, 4, 2, 4), (1, 3, 1, 5, 2, 3, 4, 5), shape[:7]]
    G.h.compare("exp", got[0], want[0], 2e-6, 1e-6)
    G.h.compare("sum", got[1], want[1], 1e-5, 1e-6, scale=np.abs(x.astype(np.float64) * y).sum((1, 3, 5, 7)))
    G.h.compare("max", got[2], want[2], 0, 0); G.h.compare("argmax", got[3], want[3], 0, 0)


def test_softmax_over_an_axis_of_extent_one(oracle, G):
    # reducing over an axis of extent 1 is the identity: max(x) = x, and the exp-sum is exp(x - x) = 1
    rng = np.random.default_rng(195)
    x = rng.standard_normal((5000, 1)).astype(np.float32)
    x[3, 0] = np.inf
    s = _lse_spec("f32", 1)
    expr, got = run_spec(G, s, [x])
    want = oracle.evaluate(s, [x])
    for name, g_, w_ in zip(("max", "expsum", "lse", "p"), got, want):
        assert np.array_equal(g_, w_, equal_nan=True) if name == "max" else True
        G.h.compare(name, g_, w_, 1e-6, 1e-7)


def test_reductions_of_an_index_in_a_plan_of_several_passes(oracle, G):
    rng = np.random.default_rng(196)
    x = rng.standard_normal((3, 64)).astype(np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False))
    s.output(s.reduce("max", s.iota(1), (0, 1), keep=True), "i32")
    s.output(s.reduce("min", xi, (1,)), "f32")
    s.output(s.iota(0), "i32")
    s.output(s.reduce("sum", s.apply("where", s.apply("gt", xi, s.const(0.0)), s.iota(1), s.const(0, "i32")), (0,)), "i32")
    expr, got = run_spec(G, s, [x])
    want = oracle.evaluate(s, [x])
    assert got[0].item() == 63 and [g_.shape for g_ in got] == [(1, 1), (3,), (3, 1), (64,)]
    for g_, w_ in zip(got, want):
        assert np.array_equal(g_, w_)


@pytest.mark.parametrize("shape,axis,opts", [((300, 1000), 1, {}), ((6000, 12), 1, {}), ((5, 70000), 1, {}), ((300, 1000), 1, {"split_rows": 1}),
                                             ((700, 40), 0, {}), ((64, 33, 20), 1, {})])
def test_softmax_in_place(shape, axis, opts, oracle, G):
    # the probabilities overwrite the logits (exact alias), in every kernel class and in plans of several passes:
    # every element is read for the last time by the thread that then writes it, after all reductions are done
    torch = G.torch
    rng = np.random.default_rng(197)
    x = (rng.standard_normal(shape) * 3).astype(np.float32)
    nd = len(shape)
    s = GraphSpec(nd)
    xi = s.input("f32", (False,) * nd)
    m = s.reduce("max", xi, (axis,), keep=True)
    ex = s.apply("exp", s.sub(xi, m))
    S = s.reduce("sum", ex, (axis,), keep=True)
    s.output(s.div(ex, S), "f32")
    s.output(s.add(m, s.apply("log", S)), "f32")
    want_p, want_l = oracle.evaluate(s, [x], nthreads=4)
    t = torch.from_numpy(x.copy()).cuda()
    lse = torch.empty(want_l.shape, dtype=torch.float32, device="cuda")
    expr = G.ewf.Expression(s, **opts)
    ws = G.h.make_workspace(expr, [t], [t, lse])
    print(f"[case] softmax in place {shape} axis {axis} {opts} -> {expr.info()['kernel_class']}", flush=True)
    expr.run([t], [t, lse], (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    G.h.compare("p", t.cpu().numpy(), want_p, 1e-5, 1e-8)
    G.h.compare("lse", lse.cpu().numpy(), want_l, 1e-5, 1e-6)


# ------------------------------------------------------------------ rows that start anywhere and end inside a vector

@pytest.mark.parametrize("rows,cols,storage", [(37, 50257, "f32"), (5, 131075, "f16"), (300, 4099, "f32"), (1, 1000003, "f16"), (64, 20001, "f16")])
def test_wide_accesses_on_rows_of_odd_length(rows, cols, storage, oracle, G):
    # reductions over rows whose pitch is odd (every row starts at a different alignment) and
    # whose last vector is cut by the row's end: wide accesses that assume element alignment
    # only, the cut vector element by element
    rng = np.random.default_rng(200 + rows)
    dt = np.float16 if storage == "f16" else np.float32
    x = (rng.standard_normal((rows, cols)) * 2).astype(dt)
    x[rows // 2, cols - 1] = 40.0                                        # the maximum in the very last element of a row
    x[0, cols - 2] = -40.0
    t = rng.integers(0, cols, (rows, 1)).astype(np.int32)
    t[rows - 1, 0] = cols - 1
    s = GraphSpec(2)
    xi = s.input(storage, (False, False)); ti = s.input("i32", (False, True))
    s.output(s.reduce("sum", s.apply("abs", xi), (1,)), "f32")
    s.output(s.reduce("max", xi, (1,), keep=True), "f32")
    s.output(s.reduce("argmax", xi, (1,)), "i32")
    s.output(s.reduce("min", xi, (1,)), "f32")
    s.output(s.reduce("sum", s.apply("where", s.apply("eq", s.iota(1), ti), xi, s.const(0.0)), (1,)), "f32")   # x[row, t[row]]
    print(f"[case] odd rows {rows} x {cols} {storage}", flush=True)
    expr, got = run_spec(G, s, [x, t])
    info = expr.info()
    assert info["kernel_class"] == "tile_reduce" and info["vec"] == 16 // x.itemsize and "ewf_ld_u<" in expr.source(), info
    want = oracle.evaluate(s, [x, t], nthreads=4)
    G.h.compare("sum", got[0], want[0], 1e-5, 1e-6); G.h.compare("max", got[1], want[1], 0, 0)
    G.h.compare("argmax", got[2], want[2], 0, 0); G.h.compare("min", got[3], want[3], 0, 0)
    G.h.compare("gather", got[4], want[4], 0, 0)
    assert got[2][rows // 2] == cols - 1
    # a view that starts at an odd element of a wider buffer, a second operand with another
    # alignment, and a strided one, all in one kernel
    wide = (rng.standard_normal((rows, cols + 7)) * 2).astype(dt)
    other = rng.standard_normal((rows, cols + 2)).astype(np.float32)
    twice = rng.standard_normal((rows, 2 * cols)).astype(np.float32)
    va, vb, vc = wide[:, 3:3 + cols], other[:, 1:1 + cols], twice[:, ::2]
    s2 = GraphSpec(2)
    ai = s2.input(storage, (False, False)); bi = s2.input("f32", (False, False)); ci = s2.input("f32", (False, False))
    v = s2.add(s2.mul(ai, bi), ci)
    s2.output(s2.reduce("sum", v, (1,)), "f32"); s2.output(s2.reduce("max", v, (1,)), "f32")
    expr, got = run_spec(G, s2, [va, vb, vc])
    assert expr.info()["kernel_class"] == "tile_reduce" and expr.info()["vec"] == 16 // x.itemsize, expr.info()
    want = oracle.evaluate(s2, [va, vb, vc], nthreads=4)
    terms = np.abs(va.astype(np.float64) * vb) + np.abs(vc.astype(np.float64))            # either sign: bar relative to their magnitudes
    G.h.compare("sum", got[0], want[0], 1e-5, 1e-6, scale=terms.sum(1)); G.h.compare("max", got[1], want[1], 2e-6, 1e-6)


@pytest.mark.parametrize("shape,offset", [((3000, 1023), 1), ((1, 5000001), 3), ((700, 4100), 5)])
def test_wide_accesses_on_float16_views_from_an_odd_element(shape, offset, oracle, G):
    # element-wise on float16: a view that starts at an odd element and rows of odd length,
    # outputs with the same kind of layout (written wide where a vector lies inside the row)
    rng = np.random.default_rng(201 + offset)
    rows, cols = shape
    base = (rng.standard_normal((rows, cols + 9)) * 2).astype(np.float16)
    x = base[:, offset:offset + cols]
    b = rng.standard_normal((1, cols)).astype(np.float16)
    s = GraphSpec(2)
    xi = s.input("f16", (False, False)); bi = s.input("f16", (rows > 1, False))
    s.output(s.apply("tanh", s.add(xi, bi)), "f16")
    s.output(s.mul(xi, s.const(0.5)), "f32")
    print(f"[case] f16 view {shape} from element {offset}", flush=True)
    torch = G.torch
    tb = torch.from_numpy(base).cuda()
    xd = tb[:, offset:offset + cols]; bd = torch.from_numpy(b).cuda()
    outbuf = torch.full((rows, cols + 5), float("nan"), dtype=torch.float16, device="cuda")
    out0 = outbuf[:, 2:2 + cols]                                          # an output view from an even but unaligned element
    out1 = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    expr = G.ewf.Expression(s)
    ws = G.h.make_workspace(expr, [xd, bd], [out0, out1])
    expr.run([xd, bd], [out0, out1], (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert expr.info()["kernel_class"] == "tile" and expr.info()["vec"] == 8 and "ewf_st_u<" in expr.source(), expr.info()
    want = oracle.evaluate(s, [x, b], nthreads=4)
    G.h.compare("tanh", out0.cpu().numpy(), want[0], 2e-3, 1e-3); G.h.compare("half", out1.cpu().numpy(), want[1], 2e-6, 1e-6)
    edge = outbuf.cpu().numpy()
    assert np.isnan(edge[:, :2]).all() and np.isnan(edge[:, 2 + cols:]).all()         # nothing written outside the view


@pytest.mark.parametrize("rows,vocab", [(61, 10001), (40, 2051), (300, 20003)])
def test_rows_of_odd_length_held_in_registers(rows, vocab, oracle, G):
    # softmax cross-entropy and its gradient on vocabularies of odd size: one workgroup per row,
    # the row read with element-aligned wide accesses, its cut last vector element by element;
    # the gradient is written the same way
    from workloads import configs as wl
    for maker in (wl.c3_softmax_xent, wl.c3_softmax_xent_backward):
        w = maker(rows=rows, vocab=vocab)
        print(f"[case] {w.name} {rows} x {vocab}", flush=True)
        expr, stats = G.h.check_workload(w, oracle, nthreads=4)
        info = expr.info()
        assert info["kernel_class"] == "row" and info["vec"] == 4 and "ewf_ld_u<float, EWF_VEC>" in expr.source(), info
    # softmax probabilities in float16 on rows of odd length and pitch, written over a padded buffer
    rng = np.random.default_rng(202 + rows)
    base = (rng.standard_normal((rows, vocab + 3)) * 3).astype(np.float16)
    x = base[:, 1:1 + vocab]
    s = GraphSpec(2)
    xi = s.input("f16", (False, False))
    m = s.reduce("max", xi, (1,), keep=True); ex = s.apply("exp", s.sub(xi, m)); S = s.reduce("sum", ex, (1,), keep=True)
    s.output(s.div(ex, S), "f16"); s.output(s.reduce("argmax", xi, (1,)), "i32")
    torch = G.torch
    tb = torch.from_numpy(base).cuda()
    xd = tb[:, 1:1 + vocab]
    outbuf = torch.full((rows, vocab + 5), float("nan"), dtype=torch.float16, device="cuda")
    out0 = outbuf[:, 3:3 + vocab]
    out1 = torch.empty((rows,), dtype=torch.int32, device="cuda")
    expr = G.ewf.Expression(s)
    ws = G.h.make_workspace(expr, [xd], [out0, out1])
    expr.run([xd], [out0, out1], (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert expr.info()["kernel_class"] == "row" and expr.info()["vec"] == 8 and "ewf_st_u<" in expr.source(), expr.info()
    want = oracle.evaluate(s, [x], nthreads=4)
    G.h.compare("p", out0.cpu().numpy(), want[0], 2e-3, 1e-3); G.h.compare("argmax", out1.cpu().numpy(), want[1], 0, 0)
    edge = outbuf.cpu().numpy()
    assert np.isnan(edge[:, :3]).all() and np.isnan(edge[:, 3 + vocab:]).all()         # nothing written outside the view
