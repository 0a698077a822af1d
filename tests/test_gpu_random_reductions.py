"""GPU parity on randomly drawn reduction workloads at sizes where the planner leaves the small-problem
paths: many short rows (several rows per wavefront), softmax chains with and without an arg-max,
row normalisation, and sums / minima over any set of axes of tensors of about a million elements
(column kernels, lanes over an outer index, reductions taken in two steps)."""
import numpy as np
import pytest

from workloads import GraphSpec

pytestmark = pytest.mark.gpu


def _ctx():
    import torch
    import tests.harness as h
    from paper_1605_02688_amd import ewf

    class Ctx:
        pass
    G = Ctx(); G.torch, G.h, G.ewf = torch, h, ewf
    return G


def _check(G, oracle, tag, s, inputs, tols):
    import tests.test_gpu_ops_and_layouts as T
    want = oracle.evaluate(s, inputs, nthreads=4)
    expr, got = T.run_spec(G, s, inputs)
    info = expr.info()
    klass = info["kernel_class"]
    if klass == "multi":
        klass += ":" + "+".join(expr.info(i)["kernel_class"] for i in range(info["grid_blocks"]))
    print(f"[ok-so-far] {tag} -> {klass}", flush=True)
    for k, (g_, w_, tol) in enumerate(zip(got, want, tols)):
        rtol, atol = tol[:2]
        if rtol == 0 and atol == 0:
            assert np.array_equal(g_, w_, equal_nan=True), f"{tag} output {k}: {np.argwhere(g_ != w_)[:3].tolist()}"
        else:               # (a third entry: the sum of the magnitudes of a sum's terms, which the bar is then relative to)
            G.h.compare(f"{tag}.out{k}", g_, w_, rtol, atol, scale=tol[2] if len(tol) > 2 else None)


@pytest.mark.parametrize("seed", range(24))
def test_random_short_rows(seed, oracle):
    G = _ctx()
    rng = np.random.default_rng(31000 + seed)
    rows = int(rng.integers(4096, 12000))
    cols = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 24, 31, 32, 48, 64, 100, 128]))
    storage = "f16" if rng.integers(0, 3) == 0 else "f32"
    dt = np.float16 if storage == "f16" else np.float32
    pad = int(rng.choice([0, 0, 1, 4, 8]))
    wide = (rng.standard_normal((rows, cols + pad)) * 2).astype(dt)
    x = wide[:, :cols] if pad else wide
    t = rng.integers(0, cols, (rows, 1)).astype(np.int32)
    s = GraphSpec(2)
    xi = s.input(storage, (False, False)); ti = s.input("i32", (False, True))
    tols = []
    kind = int(rng.integers(0, 4))
    if kind == 0:                                            # plain reductions
        s.output(s.reduce("sum", xi, (1,)), "f32"); tols.append((1e-5, 1e-6, np.abs(x.astype(np.float64)).sum(1)))
        s.output(s.reduce("max", xi, (1,)), "f32"); tols.append((0, 0))
        s.output(s.reduce("argmax", xi, (1,), keep=True), "i32"); tols.append((0, 0))
    elif kind == 1:                                          # softmax probabilities and log-sum-exp
        m = s.reduce("max", xi, (1,), keep=True); ex = s.apply("exp", s.sub(xi, m)); S = s.reduce("sum", ex, (1,), keep=True)
        s.output(s.div(ex, S), storage); tols.append((1e-5, 1e-8) if storage == "f32" else (2e-3, 1e-3))
        s.output(s.add(m, s.apply("log", S)), "f32"); tols.append((1e-5, 1e-6))
    elif kind == 2:                                          # cross-entropy with arg-max and mean
        m = s.reduce("max", xi, (1,), keep=True); ex = s.apply("exp", s.sub(xi, m)); S = s.reduce("sum", ex, (1,), keep=True)
        xt = s.reduce("sum", s.apply("where", s.apply("eq", s.iota(1), ti), xi, s.const(0.0)), (1,), keep=True)
        loss = s.sub(s.add(m, s.apply("log", S)), xt)
        s.output(loss, "f32"); tols.append((1e-5, 1e-6))
        s.output(s.reduce("argmax", xi, (1,)), "i32"); tols.append((0, 0))
        s.output(s.div(s.reduce("sum", loss, (0,)), s.const(float(rows))), "f32"); tols.append((1e-5, 1e-6))
    else:                                                    # mean and variance along the row, normalised output
        inv = s.const(1.0 / cols)
        mean = s.mul(s.reduce("sum", xi, (1,), keep=True), inv)
        cen = s.sub(xi, mean)
        var = s.mul(s.reduce("sum", s.apply("sqr", cen), (1,), keep=True), inv)
        s.output(s.div(cen, s.apply("sqrt", s.add(var, s.const(1e-3)))), "f32"); tols.append((1e-5, 1e-6))
        s.output(var, "f32"); tols.append((1e-5, 1e-6))
    tag = f"rows seed {seed}: {rows} x {cols} {storage} padded by {pad}, kind {kind}"
    print(f"[case] {tag}", flush=True)
    _check(G, oracle, tag, s, [x, t], tols)


@pytest.mark.parametrize("seed", range(24))
def test_random_axis_masks(seed, oracle):
    G = _ctx()
    rng = np.random.default_rng(41000 + seed)
    nd = int(rng.integers(3, 5))
    dims = [int(rng.choice([2, 3, 4, 8, 16, 33, 64, 100])) for _ in range(nd)]
    big = int(rng.integers(0, nd))
    dims[big] = max(dims[big], int(1.2e6 / max(1, np.prod(dims) // dims[big])))
    dims = [min(d, 200000) for d in dims]
    if np.prod(dims) > 4e6:
        dims[big] = max(2, int(4e6 / (np.prod(dims) // dims[big])))
    axes = tuple(sorted(rng.choice(nd, size=int(rng.integers(1, nd)), replace=False).tolist()))
    y = rng.uniform(0.5, 1.5, dims).astype(np.float32) * np.where(rng.random(dims) < 0.5, -1, 1).astype(np.float32)
    s = GraphSpec(nd)
    yi = s.input("f32", (False,) * nd)
    s.output(s.reduce("sum", yi, axes), "f32"); s.output(s.reduce("min", yi, axes, keep=True), "f32")
    tols = [(1e-5, 1e-6, np.abs(y.astype(np.float64)).sum(axes)), (0, 0)]      # terms of either sign
    if rng.integers(0, 2):
        s.output(s.apply("abs", yi), "f32"); tols.append((0, 0))
    tag = f"axes seed {seed}: {dims} reduced over {axes}"
    print(f"[case] {tag}", flush=True)
    _check(G, oracle, tag, s, [y], tols)


@pytest.mark.parametrize("seed", range(32))
def test_random_column_plans_at_streaming_size(seed, oracle):
    """Reductions over axes other than the innermost one, on half a million to four million
    elements: past the small-problem shapes a thread keeps several loads in flight, short reduced
    axes with few columns put outer indices on the spare lanes (several per thread when rows are
    few), finishing threads write vectors, and element-wise outputs change the tile shape."""
    G = _ctx()
    rng = np.random.default_rng(91000 + seed)
    nd = int(rng.integers(2, 5))
    if seed % 3 == 0:                                        # a short reduced axis next to a few columns
        nd = max(nd, 3)
        shape = [int(rng.choice([2, 3, 5, 16])) for _ in range(nd - 3)] + [int(rng.choice([20011, 70001, 250007])),
                 int(rng.choice([2, 3, 4, 8, 16])), int(rng.choice([4, 8, 16, 24]))]
        while np.prod(shape) > 3e6:
            shape[nd - 3] //= 2
        axes = (nd - 2,) if rng.integers(0, 2) or nd == 3 else (0, nd - 2)
    else:
        inner = int(rng.choice([8, 16, 40, 64, 100, 224, 256, 520, 1024]))
        shape = [int(rng.choice([2, 3, 4, 7, 16, 33, 64, 200, 1000, 5001])) for _ in range(nd - 1)] + [inner]
        target = int(rng.choice([6e5, 1.5e6, 4e6]))
        while np.prod(shape) > target:
            k = int(np.argmax(shape[:-1])); shape[k] = max(2, shape[k] // 2)
        while np.prod(shape) < target / 3:
            k = int(rng.integers(nd - 1)); shape[k] = shape[k] * 2 + 1
        axes = tuple(sorted(rng.choice(nd - 1, size=int(rng.integers(1, nd)), replace=False).tolist()))
    storage = "f16" if rng.integers(0, 3) == 0 else "f32"
    dt = np.float16 if storage == "f16" else np.float32
    x = rng.uniform(0.25, 2.0, shape).astype(dt)
    if rng.integers(0, 3) == 0:                              # rows with a pitch
        big = rng.uniform(0.25, 2.0, [e + (8 if d == nd - 1 else 1) for d, e in enumerate(shape)]).astype(dt)
        x = big[tuple(slice(0, e) for e in shape)]
    s = GraphSpec(nd)
    inputs = [x]
    xi = s.input(storage, (False,) * nd)
    v = xi
    if rng.integers(0, 2):                                   # constant along the reduced axes: loaded once per tile
        bc = tuple(d in axes for d in range(nd))
        inputs.append(rng.uniform(-0.5, 0.5, [1 if d in axes else shape[d] for d in range(nd)]).astype(np.float32))
        v = s.add(v, s.input("f32", bc))
    if rng.integers(0, 2) and len(axes) < nd:                # varies along the reduced axes only
        bc = tuple(d not in axes for d in range(nd))
        inputs.append(rng.uniform(0.5, 1.5, [shape[d] if d in axes else 1 for d in range(nd)]).astype(np.float32))
        v = s.mul(v, s.input("f32", bc))
    if rng.integers(0, 2):
        v = s.apply(["tanh", "sqrt", "sqr", "sigmoid"][int(rng.integers(4))], v)
    tols = []
    if rng.integers(0, 2):
        s.output(s.apply("max", s.const(0.6), v), storage); tols.append((2e-6, 1e-6) if storage == "f32" else (2e-3, 1e-3))
    keep = bool(rng.integers(0, 2))
    for _ in range(int(rng.integers(1, 4))):
        r = int(rng.integers(0, 5))
        if r == 0: s.output(s.reduce("sum", v, axes, keep=keep), "f32"); tols.append((1e-5, 1e-6))
        elif r == 1: s.output(s.reduce("max", v, axes, keep=keep), "f32"); tols.append((2e-6, 1e-6))
        elif r == 2: s.output(s.reduce("min", xi, axes, keep=keep), storage); tols.append((0, 0))
        elif r == 3: s.output(s.apply("log", s.reduce("sum", s.apply("sqr", v), axes, keep=keep)), "f32"); tols.append((1e-5, 1e-6))
        else:
            s.output(s.reduce("argmax", xi, (axes[-1],), keep=keep), "i32"); tols.append((0, 0))
            break
    _check(G, oracle, f"columns seed{seed} {storage} shape{shape} axes{axes}", s, inputs, tols)


@pytest.mark.parametrize("seed", range(16))
def test_random_column_plans_with_few_or_odd_columns(seed, oracle):
    """Sums, maxima and arg-maxima over outer axes of tensors whose innermost axis has 3 to 1001
    elements, an odd count: only narrow accesses are possible, several rows are kept in flight."""
    G = _ctx()
    rng = np.random.default_rng(95000 + seed)
    nd = int(rng.integers(2, 4))
    cols = int(rng.choice([3, 5, 7, 13, 21, 49, 51, 255, 1001]))
    if nd == 2:
        shape = [int(rng.integers(600000, 2500000)) // cols, cols]; axes = (0,)
    else:
        mid = int(rng.choice([2, 3, 7, 16, 50]))
        shape = [int(rng.integers(600000, 2500000)) // cols // mid, mid, cols]
        axes = (0,) if rng.integers(0, 2) else ((1,) if rng.integers(0, 2) else (0, 1))
    storage = "f16" if rng.integers(0, 2) else "f32"
    x = rng.uniform(0.25, 2.0, shape).astype(np.float16 if storage == "f16" else np.float32)
    if rng.integers(0, 3) == 0:                              # rows with a pitch, from an odd element
        big = rng.uniform(0.25, 2.0, shape[:-1] + [cols + 3]).astype(x.dtype); x = big[..., 1:1 + cols]
    s = GraphSpec(nd)
    xi = s.input(storage, (False,) * nd)
    s.output(s.reduce("sum", xi, axes), "f32"); s.output(s.reduce("max", xi, axes, keep=True), storage)
    tols = [(1e-5, 1e-6), (0, 0)]
    if len(axes) == 1:
        s.output(s.reduce("argmax", xi, axes), "i32"); tols.append((0, 0))
    _check(G, oracle, f"narrow columns seed{seed} {storage} shape{shape} axes{axes}", s, [x], tols)


@pytest.mark.parametrize("seed", range(32))
def test_random_row_reductions_followed_by_reductions_over_the_rows(seed, oracle):
    """Per-row sums, extremes, arg-max and log-sum-exp, then a sum / maximum / minimum of those
    over the rows: rows held by a workgroup, several rows per wavefront, rows split over
    workgroups with the second reduction folded by the finish kernel (a thread or a wavefront per
    row), with NaN and infinities in some inputs."""
    import tests.test_gpu_ops_and_layouts as T
    G = _ctx()
    rng = np.random.default_rng(515000 + seed)
    mode = seed % 4
    if mode == 0: rows, cols = int(rng.choice([1, 3, 17, 100])), int(rng.choice([40000, 70001, 200000]))
    elif mode == 1: rows, cols = int(rng.choice([300, 600, 1500])), int(rng.choice([9000, 20000, 33000]))
    elif mode == 2: rows, cols = int(rng.choice([5, 64, 700])), int(rng.choice([7, 100, 1003, 4096]))
    else: rows, cols = int(rng.choice([2000, 9000])), int(rng.choice([600, 2048]))
    storage = "f16" if rng.integers(0, 4) == 0 else "f32"
    x = (rng.standard_normal((rows, cols)) * 2).astype(np.float16 if storage == "f16" else np.float32)
    if rng.integers(0, 3) == 0 and rows > 2:
        x[int(rng.integers(rows)), int(rng.integers(cols))] = np.nan
        x[int(rng.integers(rows)), int(rng.integers(cols))] = -np.inf
    s = GraphSpec(2)
    xi = s.input(storage, (False, False))
    affine = bool(rng.integers(0, 2))
    f = s.add(s.mul(xi, s.const(0.5)), s.const(0.25)) if affine else xi
    fx = x.astype(np.float64) * 0.5 + 0.25 if affine else x.astype(np.float64)
    per_row, tols = [], []
    kinds = rng.choice(["sum", "max", "argmax", "lse", "min", "sumsq"], size=int(rng.integers(1, 4)), replace=False).tolist()
    for k in kinds:
        if k == "sum":
            v = s.reduce("sum", f, (1,)); per_row.append((v, (0,), len(tols))); s.output(v, "f32")
            mag = np.abs(fx).sum(axis=1)
            tols.append((1e-5, 1e-6, np.where(np.isfinite(mag), mag, 0.0)))
        elif k in ("max", "min"):
            v = s.reduce(k, f, (1,)); per_row.append((v, (0,), len(tols))); s.output(v, "f32"); tols.append((2e-6, 1e-6))
        elif k == "argmax":
            v = s.reduce("argmax", f, (1,)); per_row.append((s.cast(v, "f32"), (0,), len(tols))); s.output(v, "i32"); tols.append((0, 0))
        elif k == "sumsq":
            v = s.reduce("sum", s.mul(f, f), (1,)); per_row.append((v, (0,), len(tols))); s.output(v, "f32"); tols.append((1e-5, 1e-6))
        else:
            m = s.reduce("max", f, (1,), keep=True)
            lse = s.add(m, s.apply("log", s.reduce("sum", s.apply("exp", s.sub(f, m)), (1,), keep=True)))
            per_row.append((lse, (0, 1), len(tols))); s.output(lse, "f32"); tols.append((1e-5, 1e-6))
    for _ in range(int(rng.integers(1, 3))):
        v, axes, src = per_row[int(rng.integers(len(per_row)))]
        op = ["sum", "max", "min"][int(rng.integers(3))]
        r = s.reduce(op, v, axes)
        div = float(rows) if rng.integers(0, 2) else 1.0
        if div != 1.0:
            r = s.div(r, s.const(div))
        s.output(r, "f32")
        # the bar for reductions; a sum over the rows relative to the sum of the magnitudes of the
        # per-row values (each of which carries its own rounding error)
        tols.append((1e-5, 1e-6, ("rows", src, div)) if op == "sum" else (1e-5, 1e-6))
    opts = [{}, {}, {"split_rows": 1}, {"split_rows": 2}][int(rng.integers(4))]
    tag = f"seed={seed} rows={rows} cols={cols} {storage} kinds={kinds} opts={opts}"
    print(f"[case] {tag}", flush=True)
    try:
        expr, got = T.run_spec(G, s, [x], **opts)
    except G.ewf.EwfError as e:
        assert e.status == G.ewf.EUNSUPPORTED, e         # an option that does not fit is refused, never run wrongly
        expr, got = T.run_spec(G, s, [x])
    want = oracle.evaluate(s, [x], nthreads=8)
    for k, (g_, w_, tol) in enumerate(zip(got, want, tols)):
        if tol[:2] == (0, 0):
            assert np.array_equal(g_, w_), f"{tag} output {k}"
            continue
        scale = tol[2] if len(tol) > 2 else None
        if isinstance(scale, tuple):
            terms = np.abs(want[scale[1]].astype(np.float64))
            total = np.where(np.isfinite(terms), terms, 0.0).sum() / scale[2]
            scale = np.maximum(total, np.abs(np.where(np.isfinite(w_), w_, 0.0)))
        elif scale is not None:
            scale = np.maximum(scale, np.abs(np.where(np.isfinite(w_), w_, 0.0))).reshape(w_.shape)
        G.h.compare(f"{tag}.out{k}", g_, w_, tol[0], tol[1], scale=scale)


@pytest.mark.parametrize("seed", range(40))
def test_random_argmax_over_several_axes(seed, oracle):
    """The position of the first maximum in the row-major order of any set of reduced axes, on
    contiguous, permuted and sliced inputs of every storage type, with many ties, NaN and
    infinities; exact."""
    import tests.test_gpu_ops_and_layouts as T
    G = _ctx()
    rng = np.random.default_rng(880000 + seed)
    nd = int(rng.integers(2, 5))
    shape = [int(rng.choice([1, 2, 3, 5, 8, 17, 64])) for _ in range(nd)]
    if seed % 2:
        shape[int(rng.integers(nd))] = int(rng.choice([257, 1000, 4099, 20000]))
    while np.prod(shape) > 4e6:
        shape[int(np.argmax(shape))] //= 2
    storage = ["f32", "f16", "i32"][seed % 3]
    dt = {"f32": np.float32, "f16": np.float16, "i32": np.int32}[storage]
    x = rng.integers(-4, 5, shape).astype(dt)
    if storage != "i32" and rng.integers(0, 2) and x.size > 4:
        flat = x.reshape(-1)
        flat[int(rng.integers(x.size))] = np.nan
        flat[int(rng.integers(x.size))] = np.inf
    style = int(rng.integers(0, 3))
    if style == 1:
        perm = rng.permutation(nd)
        x = np.ascontiguousarray(x.transpose(perm)).transpose(np.argsort(perm))
    elif style == 2:
        big = np.zeros([e + 2 for e in shape], dt)
        inner = tuple(slice(1, 1 + e) for e in shape)
        big[inner] = x
        x = big[inner]
    axes = tuple(sorted(rng.choice(nd, size=int(rng.integers(1, nd + 1)), replace=False).tolist()))
    keep = bool(rng.integers(0, 2))
    s = GraphSpec(nd)
    xi = s.input(storage, (False,) * nd)
    s.output(s.reduce("argmax", xi, axes, keep=keep), "i32")
    s.output(s.reduce("max", xi, axes, keep=keep), "i32" if storage == "i32" else "f32")
    opts = [{}, {}, {}, {"force_scalar": 1}, {"block_threads": 64}, {"tile_elems": 512}, {"max_blocks": 5}, {"plain_extremes": 1}][int(rng.integers(8))]
    print(f"[case] seed={seed} shape={shape} {storage} style={style} axes={axes} keep={keep} opts={opts}", flush=True)
    expr, got = T.run_spec(G, s, [x], **opts)
    want = oracle.evaluate(s, [x], nthreads=8)
    assert np.array_equal(got[0], want[0]), (expr.info()["kernel_class"], np.argwhere(got[0] != want[0])[:3].tolist())
    assert np.array_equal(got[1], want[1], equal_nan=True)


@pytest.mark.parametrize("shape,axes", [((8, 700, 3000), (1, 2)), ((700, 8, 3000), (0, 2)), ((3000, 700, 8), (0, 1)), ((40, 50, 60, 70), (0, 1, 2, 3))])
def test_argmax_over_several_axes_of_large_tensors(shape, axes, oracle):
    """Groups that span many tiles: the partial results carry flattened positions and are folded
    by value, then by position."""
    import tests.test_gpu_ops_and_layouts as T
    G = _ctx()
    rng = np.random.default_rng(4242)
    x = rng.integers(-50, 51, shape).astype(np.float32)
    s = GraphSpec(len(shape))
    xi = s.input("f32", (False,) * len(shape))
    s.output(s.reduce("argmax", xi, axes), "i32")
    s.output(s.reduce("max", xi, axes), "f32")
    print(f"[case] argmax shape={shape} axes={axes}", flush=True)
    expr, got = T.run_spec(G, s, [x])
    kept = [d for d in range(len(shape)) if d not in axes]
    moved = np.transpose(x, kept + list(axes)).reshape([shape[d] for d in kept] + [-1])
    want = oracle.evaluate(s, [x], nthreads=16)
    assert np.array_equal(want[0], np.argmax(moved, axis=-1).astype(np.int32))       # the oracle against numpy, at this size too
    assert np.array_equal(got[0], want[0]) and np.array_equal(got[1], want[1])
