"""ewf_run allocates nothing, synchronises nothing and records no memset, so a launch-bound
inner loop (the LSTM cell applied step after step, the body of the paper's Scan, section 2.1.4)
can be captured into a HIP graph and replayed.  Replays are checked against the eager results
several times, with eager work and synchronisations in between, and the eager recurrence
against the oracle."""
import numpy as np
import pytest

from workloads import configs as wl

pytestmark = pytest.mark.gpu


def test_lstm_steps_in_a_captured_graph(oracle):
    import torch
    import tests.harness as h
    from paper_1605_02688_amd import ewf

    T, B, Hd = 12, 16, 256
    w = wl.c2_lstm_cell(batch=B, hidden=Hd)
    rng = np.random.default_rng(190)
    P_all = rng.standard_normal((T, B, 4 * Hd)).astype(np.float32)
    bias = w.buffers[1]
    c0 = w.buffers[2]

    expr = ewf.Expression(w.spec)
    dP = torch.from_numpy(P_all).cuda()
    dbias = torch.from_numpy(bias).cuda()
    cbuf = [torch.from_numpy(c0).cuda(), torch.empty((B, Hd), dtype=torch.float32, device="cuda")]
    hbuf = torch.empty((T, B, Hd), dtype=torch.float32, device="cuda")

    def step_tensors(t):
        Pt = dP[t]
        ins = [Pt[:, k * Hd:(k + 1) * Hd] for k in range(4)] + [dbias[:, k * Hd:(k + 1) * Hd] for k in range(4)] + [cbuf[t % 2]]
        outs = [hbuf[t], cbuf[(t + 1) % 2]]
        return ins, outs

    def run_all(stream):
        for t in range(T):
            ins, outs = step_tensors(t)
            expr.run(ins, outs, (), None, stream)

    c_start = cbuf[0].clone()
    # eager (also plans, compiles and loads the kernel before any capture)
    run_all(torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    eager_h = hbuf.clone(); eager_c = cbuf[T % 2].clone()

    # oracle: the same recurrence on the host
    c = c0.copy()
    for t in range(T):
        ins = [np.ascontiguousarray(P_all[t][:, k * Hd:(k + 1) * Hd]) for k in range(4)]
        ins += [np.ascontiguousarray(bias[:, k * Hd:(k + 1) * Hd]) for k in range(4)] + [c]
        hh, c = oracle.evaluate(w.spec, ins)
        h.compare(f"h[{t}]", eager_h[t].cpu().numpy(), hh, 2e-6, 1e-6)
    h.compare("c[T]", eager_c.cpu().numpy(), c, 2e-6, 1e-6)

    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        cbuf[0].copy_(c_start)
        with torch.cuda.graph(graph, stream=side):
            run_all(torch.cuda.current_stream().cuda_stream)
    torch.cuda.current_stream().wait_stream(side)
    for replay in range(4):
        cbuf[0].copy_(c_start)
        hbuf.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(hbuf, eager_h), f"replay {replay}: h differs from the eager run"
        assert torch.equal(cbuf[T % 2], eager_c), f"replay {replay}: c differs from the eager run"
        # eager work between replays
        scratch = torch.randn(1 << 16, device="cuda").sum().item()
        assert np.isfinite(scratch)

    # the same steps as one prepared sequence: the loop over the steps runs inside the library
    calls = []
    for t in range(T):
        ins, outs = step_tensors(t)
        calls.append(expr.bind(ins, outs, (), None, torch.cuda.current_stream().cuda_stream))
    seq = ewf.CallSequence(calls)
    for _ in range(2):
        cbuf[0].copy_(c_start)
        hbuf.zero_()
        seq.launch()
        torch.cuda.synchronize()
        assert torch.equal(hbuf, eager_h) and torch.equal(cbuf[T % 2], eager_c)
    # and a single prepared call
    cbuf[0].copy_(c_start)
    hbuf.zero_()
    calls[0].launch()
    torch.cuda.synchronize()
    assert torch.equal(hbuf[0], eager_h[0])
