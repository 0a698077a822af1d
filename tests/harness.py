"""Shared helpers of the GPU parity tests: runs a workload through the library's C ABI binding
(device memory from `paper_1605_02688_amd.torchmem`), runs the oracle on the host arrays,
compares."""
from __future__ import annotations

import os

import numpy as np
import torch

from paper_1605_02688_amd import ewf
from workloads import configs as wl

from paper_1605_02688_amd.torchmem import alloc_outputs, device_inputs, make_workspace  # noqa: F401  (used by the tests)
from paper_1605_02688_amd.torchmem import run_workload as run_gpu  # noqa: F401


# The three bars the parity tests are held to (relative, absolute).
ELEMENTWISE, REDUCTION, HALF = (2e-6, 1e-6), (1e-5, 1e-6), (2e-3, 1e-3)


def compare(name, got, want, rtol, atol, scale=None):
    """|got - want| <= atol + rtol*|want| element by element; NaN matches NaN; exact when both
    tolerances are zero.  Returns (max abs error, max rel error).

    `scale` (an array broadcastable to the result) replaces |want| in the bar.  It is the sum of the
    magnitudes of a sum's terms: the rounding error of a floating-point sum is proportional to
    that, not to the result, which cancellation between terms of either sign can make
    arbitrarily small; where all terms share a sign the two are the same number."""
    assert got.shape == want.shape, (name, got.shape, want.shape)
    assert got.dtype == want.dtype, (name, got.dtype, want.dtype)
    if rtol == 0 and atol == 0:
        assert np.array_equal(got, want), f"{name}: integer/exact output differs at {np.argwhere(got != want)[:5]}"
        return 0.0, 0.0
    g = got.astype(np.float64); o = want.astype(np.float64)
    both_nan = np.isnan(g) & np.isnan(o)
    same_inf = np.isinf(o) & (g == o)
    err = np.where(both_nan | same_inf, 0.0, np.abs(g - o))
    mag = np.abs(np.where(np.isfinite(o), o, 0.0))
    if scale is not None:
        mag = np.broadcast_to(np.asarray(scale, np.float64), o.shape)
        assert (mag >= np.abs(np.where(np.isfinite(o), o, 0.0)) * (1 - 1e-6)).all(), f"{name}: scale below |want|"
    lim = atol + rtol * mag
    bad = ~(err <= lim)
    if os.environ.get("EWF_COMPARE_LOG"):
        # one line per comparison: the bar used, the largest error, and the share of this bar and
        # of the three stated bars that the worst element takes (for reviewing the bars)
        def share(rt, at):
            return float((err / (at + rt * mag)).max(initial=0.0))
        with open(os.environ["EWF_COMPARE_LOG"], "a") as f:
            f.write(f"{os.environ.get('PYTEST_CURRENT_TEST', '?').split(' ')[0]}\t{name}\t{rtol:g}\t{atol:g}\t"
                    f"{float(err.max(initial=0.0)):.3g}\t{share(rtol, atol):.3g}\t{share(2e-6, 1e-6):.3g}\t"
                    f"{share(1e-5, 1e-6):.3g}\t{share(2e-3, 1e-3):.3g}\n")
    if bad.any():
        idx = np.argwhere(bad)[:5]
        raise AssertionError(f"{name}: {int(bad.sum())} of {bad.size} elements out of tolerance "
                             f"(rtol={rtol}, atol={atol}); first at {idx.tolist()}: got {g[bad][:5]}, want {o[bad][:5]}")
    with np.errstate(divide="ignore", invalid="ignore"):
        rel = np.where(np.abs(o) > 0, err / np.abs(o), 0.0)
    return float(err.max(initial=0.0)), float(rel.max(initial=0.0))


def product_rtol(n):
    """Relative bar for a float32 product of n factors: every multiplication rounds (2^-24
    relative) and the errors add up in the exponent, n * 2^-24 at worst and sqrt(n) * 2^-24 as a
    random walk; four such deviations where that exceeds the stated bar for reductions."""
    return max(REDUCTION[0], 4.0 * float(n) ** 0.5 * 2.0 ** -24)


_EXACT_OPS = ("neg", "abs", "max", "min", "where", "gt", "ge", "lt", "le", "eq", "ne")


def rounding_depth(spec, value):
    """Number of rounding operations on the longest path from the leaves to `value` (selections,
    comparisons, sign changes and extreme values are exact and do not count)."""
    depth = []
    for node in spec.nodes:
        k = node[0]
        if k == "apply":
            depth.append(max(depth[a] for a in node[2]) + (0 if node[1] in _EXACT_OPS else 1))
        elif k == "cast":
            depth.append(depth[node[1]] + 1)
        elif k == "reduce":
            depth.append(depth[node[2]] + (1 if node[1] in ("sum", "prod") else 0))
        else:
            depth.append(0)
    return max(1, depth[value])


def check_workload(w, oracle, nthreads=8, **opts):
    expr, got = run_gpu(w, **opts)
    want = oracle.evaluate(w.oracle_spec or w.spec, wl.host_inputs(w), w.scalars, nthreads=nthreads)
    stats = {}
    for name, g, o, (rtol, atol) in zip(w.out_names, got, want, w.tol):
        stats[name] = compare(f"{w.name}.{name}", g, o, rtol, atol)
    return expr, stats
