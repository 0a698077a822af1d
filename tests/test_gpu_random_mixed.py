"""GPU parity on randomly generated expressions with mixed storage types (float32, float16,
int32), integer values, casts, indices, strided and permuted views, any set of reduced axes and
randomly chosen tuning options -- against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest

from workloads import GraphSpec

pytestmark = pytest.mark.gpu

OPTION_SETS = [{}, {}, {}, {}, {"force_index64": 1}, {"force_scalar": 1}, {"block_threads": 64}, {"block_threads": 1024},
               {"unroll": 1}, {"unroll": 4}, {"max_blocks": 5}, {"tile_elems": 512}, {"no_rewrite": 1}, {"no_lds_staging": 1},
               {"no_prefetch": 2}, {"xcd_remap": 1}, {"streaming": 1}]


def _view(rng, shape, dt, lo, hi):
    """A tensor of the given shape: contiguous, a slice of a larger one, a permuted one or every second element."""
    if np.issubdtype(dt, np.integer):
        gen = lambda sh: rng.integers(lo, hi, sh).astype(dt)        # noqa: E731
    else:
        gen = lambda sh: rng.uniform(lo, hi, sh).astype(dt)         # noqa: E731
    style = int(rng.integers(0, 4))
    if style == 0:
        return gen(shape)
    if style == 1:
        return gen([e + 2 for e in shape])[tuple(slice(1, 1 + e) for e in shape)]
    if style == 2:
        perm = rng.permutation(len(shape))
        return gen([shape[p] for p in perm]).transpose(np.argsort(perm))
    return gen([2 * e for e in shape])[tuple(slice(0, 2 * e, 2) for e in shape)]


def random_mixed_case(seed):
    rng = np.random.default_rng(73000 + seed)
    opts = OPTION_SETS[int(rng.integers(len(OPTION_SETS)))]
    nd = int(rng.integers(1, 5))
    full = [int(rng.choice([1, 2, 3, 5, 8, 16, 31, 64, 100])) for _ in range(nd)]
    if rng.integers(0, 2):
        full[int(rng.integers(nd))] = int(rng.choice([257, 1000, 4099]))
    while np.prod(full) > 2e6:
        full[int(np.argmax(full))] //= 2
    s = GraphSpec(nd)
    inputs, fvals, ivals = [], [], []
    for k in range(int(rng.integers(1, 4))):
        bc = tuple(bool(rng.integers(0, 4) == 0) and k > 0 for _ in range(nd))
        shp = [1 if b else e for b, e in zip(bc, full)]
        kind = int(rng.integers(0, 3))
        if kind == 2:
            inputs.append(_view(rng, shp, np.int32, -50, 50)); ivals.append(s.input("i32", bc))
        else:
            inputs.append(_view(rng, shp, np.float16 if kind == 1 else np.float32, 0.25, 2.0))
            fvals.append(s.input("f16" if kind == 1 else "f32", bc))
    if not fvals:
        fvals.append(s.cast(ivals[0], "f32"))
    if not ivals:
        ivals.append(s.cast(s.mul(fvals[0], s.const(8.0)), "i32"))
    for _ in range(int(rng.integers(2, 7))):
        r = int(rng.integers(0, 7))
        a = fvals[int(rng.integers(len(fvals)))]; b = fvals[int(rng.integers(len(fvals)))]
        if r == 0:
            fvals.append(s.apply(["tanh", "sqrt", "log1p", "sigmoid", "abs", "sqr"][int(rng.integers(6))], a))
        elif r == 1:                       # (no differences or quotients: float32 against float64 must stay comparable)
            fvals.append(s.apply(["add", "mul", "max", "min"][int(rng.integers(4))], a, s.add(b, s.const(0.5))))
        elif r == 2:
            fvals.append(s.apply("where", s.apply(["gt", "le", "eq"][int(rng.integers(3))], a, b), a, s.const(0.75)))
        elif r == 3:
            i1 = ivals[int(rng.integers(len(ivals)))]; i2 = ivals[int(rng.integers(len(ivals)))]
            ivals.append(s.apply(["add", "sub", "mul", "max", "min"][int(rng.integers(5))], i1, i2))
        elif r == 4:
            fvals.append(s.cast(ivals[int(rng.integers(len(ivals)))], "f32"))
        elif r == 5:
            ivals.append(s.apply("where", s.apply("gt", a, b), ivals[int(rng.integers(len(ivals)))], s.const(3, "i32")))
        else:
            ivals.append(s.iota(int(rng.integers(nd))))
    tols = []
    fv, iv = fvals[-1], ivals[-1]
    if rng.integers(0, 2):
        st = "f16" if rng.integers(0, 2) else "f32"
        s.output(fv, st); tols.append((2e-6, 1e-6) if st == "f32" else (2e-3, 1e-3))
    if rng.integers(0, 3) == 0:
        s.output(iv, "i32"); tols.append((0, 0))
    axes = tuple(sorted(rng.choice(nd, size=int(rng.integers(1, nd + 1)), replace=False).tolist()))
    keep = bool(rng.integers(0, 2))
    for _ in range(int(rng.integers(0 if tols else 1, 4))):
        r = int(rng.integers(0, 6))
        if r == 0:
            s.output(s.reduce("sum", fv, axes, keep=keep), "f32"); tols.append((1e-5, 1e-6))
        elif r == 1:
            s.output(s.reduce("max", fv, axes, keep=keep), "f32"); tols.append((2e-6, 1e-6))
        elif r == 2:
            s.output(s.reduce("min", fvals[0], axes, keep=keep), "f32"); tols.append((0, 0))
        elif r == 3:
            s.output(s.reduce("sum", iv, axes, keep=keep), "i32"); tols.append((0, 0))
        elif r == 4:
            s.output(s.reduce("max", iv, axes, keep=keep), "i32"); tols.append((0, 0))
        else:                              # arg-max of an input (a computed key would let rounding pick the index)
            s.output(s.reduce("argmax", ivals[0] if rng.integers(0, 2) and ivals[0] < len(inputs) else fvals[0], (axes[0],), keep=keep), "i32")
            tols.append((0, 0))
            break
    return s, inputs, tols, opts, full, axes


@pytest.mark.parametrize("seed", range(48))
def test_random_mixed_types(seed, oracle):
    import tests.harness as h
    import tests.test_gpu_ops_and_layouts as T
    import torch
    from paper_1605_02688_amd import ewf

    class Ctx:
        pass
    G = Ctx(); G.torch, G.h, G.ewf = torch, h, ewf
    s, inputs, tols, opts, full, axes = random_mixed_case(seed)
    print(f"[case] mixed seed {seed} extents {full} reduced axes {axes} options {opts} outputs {len(tols)}", flush=True)
    want = oracle.evaluate(s, inputs, nthreads=4)
    expr, got = T.run_spec(G, s, inputs, **opts)
    for k, (g_, w_, (rtol, atol)) in enumerate(zip(got, want, tols)):
        if rtol == 0 and atol == 0:
            assert np.array_equal(g_, w_, equal_nan=True), f"output {k}: {np.argwhere(g_ != w_)[:3].tolist()}"
        else:
            h.compare(f"mixed{seed}.out{k}", g_, w_, rtol, atol)
