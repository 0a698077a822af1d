"""The library driven from a plain C program (no PyTorch): tests/c_abi/c1_from_c.c is compiled
by the build step; here it runs on the GPU and its raw output files are compared with the oracle."""
import os
import subprocess

import numpy as np
import pytest

from workloads import GraphSpec

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
BINARY = os.path.join(HERE, "c_abi", "c1_from_c")


def test_c_program_through_the_abi(oracle, tmp_path):
    import tests.harness as h
    assert os.path.exists(BINARY), "build it first: python -c 'import __graft_entry__ as g; g.build()'"
    rows, cols, a = 777, 260, 0.5
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.path.join(os.path.dirname(HERE), "paper_1605_02688_amd") + ":" + env.get("LD_LIBRARY_PATH", "")
    r = subprocess.run([BINARY, str(rows), str(cols), str(a), str(tmp_path)], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "kernel_class 5" in r.stdout or "kernel_class 4" in r.stdout, r.stdout   # column sum (+ element-wise output)
    x = np.fromfile(tmp_path / "x.bin", np.float32).reshape(rows, cols)
    b = np.fromfile(tmp_path / "b.bin", np.float32).reshape(1, cols)
    y = np.fromfile(tmp_path / "y.bin", np.float32).reshape(rows, cols)
    cs = np.fromfile(tmp_path / "colsum.bin", np.float32)
    s = GraphSpec(2)
    xi = s.input("f32", (False, False)); bi = s.input("f32", (True, False)); sc = s.scalar("f32")
    yy = s.apply("tanh", s.add(s.mul(sc, xi), bi))
    s.output(yy, "f32"); s.output(s.reduce("sum", yy, (0,)), "f32")
    wy, wcs = oracle.evaluate(s, [x, b], [a])
    h.compare("y", y, wy, 2e-6, 1e-6)
    # the terms have either sign: the bar is relative to the sum of their magnitudes
    h.compare("colsum", cs, wcs, 1e-5, 1e-6, scale=np.abs(wy.astype(np.float64)).sum(0))
