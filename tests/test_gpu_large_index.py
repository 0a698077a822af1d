"""GPU parity with 64-bit element offsets: tensors of more than 2^31 elements and views whose
strides reach past 2^31 elements.  The oracle cannot walk billions of elements in seconds, so the
element-wise case is compared on sampled positions (the oracle evaluates each sample from the
input values at the same positions) and the reductions use inputs that are zero except for a few
planted powers of two, whose sums are exact in float32 at any size: a region that a kernel skips
or visits twice changes the result."""
import numpy as np
import pytest

from workloads import GraphSpec

pytestmark = pytest.mark.gpu

TWO31 = 1 << 31


@pytest.fixture()
def G():
    import gc
    import torch
    import tests.harness as h
    from paper_1605_02688_amd import ewf

    class Ctx:
        pass
    c = Ctx()
    c.torch, c.h, c.ewf = torch, h, ewf
    yield c
    gc.collect()
    torch.cuda.empty_cache()


def _run(G, spec, ins, fill=None):
    torch = G.torch
    expr = G.ewf.Expression(spec)
    outs = G.h.alloc_outputs(expr, spec, ins, fill=fill)
    ws = G.h.make_workspace(expr, ins, outs)
    expr.run(ins, outs, (), ws, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return expr, outs


def test_elementwise_over_more_than_2_to_31_elements(oracle, G):
    torch = G.torch
    n = TWO31 + 4099
    gen = torch.Generator(device="cuda"); gen.manual_seed(160502688)
    x = torch.empty(n, dtype=torch.float16, device="cuda").normal_(0.0, 1.5, generator=gen)
    s = GraphSpec(1)
    xi = s.input("f16", (False,))
    s.output(s.apply("tanh", xi), "f16")
    print(f"[case] elementwise n={n}", flush=True)
    expr, (y,) = _run(G, s, [x], fill=float("nan"))
    assert expr.info()["index_bits"] == 64
    assert not bool(torch.isnan(y).any()), "an element was never written"
    rng = np.random.default_rng(31)
    pos = np.concatenate([np.arange(0, 4096), np.arange(TWO31 - 2048, TWO31 + 2048), np.arange(n - 4099, n),
                          rng.integers(0, n, 20000)]).astype(np.int64)
    idx = torch.from_numpy(pos).cuda()
    xs = x[idx].cpu().numpy(); ys = y[idx].cpu().numpy()
    want, = oracle.evaluate(s, [xs])
    G.h.compare("tanh", ys, want, 2e-3, 1e-3)


def _plant(G, t, positions):
    """t: flat zero tensor; writes 2^j at positions[j]; returns the values planted."""
    vals = [float(1 << j) for j in range(len(positions))]
    t[G.torch.tensor(positions, device="cuda")] = G.torch.tensor(vals, dtype=t.dtype, device="cuda")
    return vals


def test_total_reduction_over_more_than_2_to_31_elements(G):
    torch = G.torch
    n = TWO31 + 4099
    x = torch.zeros(n, dtype=torch.float16, device="cuda")
    positions = [0, 1, 2047, 2048, 77777, TWO31 // 2, TWO31 - 2049, TWO31 - 1, TWO31, TWO31 + 1, TWO31 + 2048, n - 4000,
                 n - 2050, n - 2, n - 1]
    vals = _plant(G, x, positions)
    s = GraphSpec(1)
    xi = s.input("f16", (False,))
    s.output(s.reduce("sum", xi, (0,)), "f32"); s.output(s.reduce("max", xi, (0,)), "f32")
    print(f"[case] total reduction n={n}", flush=True)
    expr, (tot, mx) = _run(G, s, [x])
    assert expr.info()["index_bits"] == 64
    assert float(tot.item()) == sum(vals) and float(mx.item()) == max(vals)


def test_row_reductions_with_rows_of_2_to_30_elements(G):
    torch = G.torch
    rows, cols = 3, (1 << 30) + 5
    x = torch.zeros(rows * cols, dtype=torch.float16, device="cuda")
    in_row = [0, 1, 4095, 4096, cols // 3, cols // 2, cols - 4097, cols - 2, cols - 1]
    sums, maxs, args = [], [], []
    for r in range(rows):
        order = in_row[r:] + in_row[:r]                 # the largest value sits elsewhere in every row
        vals = _plant(G, x[r * cols:(r + 1) * cols], order)
        sums.append(sum(vals)); maxs.append(max(vals)); args.append(order[-1])
    s = GraphSpec(2)
    xi = s.input("f16", (False, False))
    s.output(s.reduce("sum", xi, (1,)), "f32"); s.output(s.reduce("max", xi, (1,)), "f32")
    s.output(s.reduce("argmax", xi, (1,)), "i32")
    print(f"[case] row reductions {rows} x {cols}", flush=True)
    expr, (rs, rm, ra) = _run(G, s, [x.view(rows, cols)])
    assert expr.info()["index_bits"] == 64
    assert rs.cpu().tolist() == sums and rm.cpu().tolist() == maxs and ra.cpu().tolist() == args


def test_column_reductions_over_more_than_2_to_31_elements(oracle, G):
    torch = G.torch
    rows, cols = (1 << 16) + 3, 1 << 15
    x = torch.zeros(rows * cols, dtype=torch.float16, device="cuda")
    cells = [(0, 0), (1, 0), (rows - 1, 0), (rows // 2, 1), (rows - 1, cols - 1), (rows - 2, cols - 1), (65536, 12345),
             (65535, 12345), (4097, 513), (rows - 3, 511), (rows - 1, 512)]
    _plant(G, x, [r * cols + c for r, c in cells])
    s = GraphSpec(2)
    xi = s.input("f16", (False, False))
    s.output(s.reduce("sum", xi, (0,)), "f32"); s.output(s.reduce("max", xi, (0,)), "f32")
    print(f"[case] column reductions {rows} x {cols}", flush=True)
    x2 = x.view(rows, cols)
    expr, (cs, cm) = _run(G, s, [x2], fill=float("nan"))
    assert expr.info()["index_bits"] == 64 and expr.info()["kernel_class"] == "col"
    # the columns that hold planted values: the oracle sums each of them whole
    touched = sorted({c for _, c in cells})
    sub = x2[:, touched].cpu().numpy()
    want_s, want_m = oracle.evaluate(s, [sub])
    got_s = cs.cpu().numpy(); got_m = cm.cpu().numpy()
    assert np.array_equal(got_s[touched], want_s) and np.array_equal(got_m[touched], want_m)
    # every other column is all zero
    rest = np.ones(cols, bool); rest[touched] = False
    assert np.all(got_s[rest] == 0.0) and np.all(got_m[rest] == 0.0)


def test_view_with_strides_past_2_to_31_elements(oracle, G):
    torch = G.torch
    rows, cols, pitch = 4097, 33, 1 << 20
    buf = torch.zeros((rows - 1) * pitch + cols, dtype=torch.float16, device="cuda")
    rng = np.random.default_rng(32)
    host = rng.standard_normal((rows, cols)).astype(np.float16)
    view = torch.as_strided(buf, (rows, cols), (pitch, 1))
    view.copy_(torch.from_numpy(host).cuda())
    s = GraphSpec(2)
    xi = s.input("f16", (False, False))
    s.output(s.apply("tanh", xi), "f16"); s.output(s.reduce("sum", xi, (1,)), "f32")
    print(f"[case] strided view {rows} x {cols}, pitch {pitch}", flush=True)
    expr, (y, rs) = _run(G, s, [view])
    assert expr.info()["index_bits"] == 64
    want_y, want_s = oracle.evaluate(s, [host])
    G.h.compare("tanh", y.cpu().numpy(), want_y, 2e-3, 1e-3)
    G.h.compare("rowsum", rs.cpu().numpy(), want_s, 1e-5, 1e-6, scale=np.abs(host.astype(np.float64)).sum(1))
