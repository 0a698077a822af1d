"""GPU parity of the five workloads against the oracle, at sizes the oracle finishes in
seconds that still span several tiles and a ragged tail."""
import numpy as np
import pytest

from workloads import configs as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import tests.harness as h
    return h


CASES = {
    "c1_full": lambda: wl.c1_affine_tanh(),
    "c1_ragged": lambda: wl.c1_affine_tanh(rows=333, cols=77),
    "c1_const_a": lambda: wl.c1_affine_tanh(rows=130, cols=256, a_form="const"),
    "c1_tensor_a": lambda: wl.c1_affine_tanh(rows=130, cols=256, a_form="tensor"),
    "c2_full": lambda: wl.c2_lstm_cell(),
    "c2_ragged": lambda: wl.c2_lstm_cell(batch=7, hidden=250),
    "c3_rows64": lambda: wl.c3_softmax_xent(rows=64, vocab=10000),
    "c3_ragged": lambda: wl.c3_softmax_xent(rows=37, vocab=1003),
    "c3_short_rows": lambda: wl.c3_softmax_xent(rows=300, vocab=40),
    "c4_small": lambda: wl.c4_bias_relu_chansum(n=4, c=64, h=112, w=112),
    "c4_ragged": lambda: wl.c4_bias_relu_chansum(n=3, c=5, h=13, w=17),
    "c5a_small": lambda: wl.c5_stress(n=2, c=256, h=56, w=56, reading="A"),
    "c5b_small": lambda: wl.c5_stress(n=2, c=256, h=56, w=56, reading="B"),
    "c5a_ragged": lambda: wl.c5_stress(n=2, c=10, h=7, w=9, reading="A"),
    "c5b_ragged_c": lambda: wl.c5_stress(n=3, c=6, h=5, w=12, reading="B", bcast="c"),
    # backward passes: the library differentiates the forward description, the oracle evaluates
    # the gradient written out by hand
    "c2b_full": lambda: wl.c2_lstm_cell_backward(),
    "c2b_ragged": lambda: wl.c2_lstm_cell_backward(batch=7, hidden=250),
    "c3b_rows64": lambda: wl.c3_softmax_xent_backward(rows=64, vocab=10000),
    "c3b_ragged": lambda: wl.c3_softmax_xent_backward(rows=37, vocab=1003),
    "c4b_small": lambda: wl.c4_bias_relu_chansum_backward(n=4, c=64, h=112, w=112),
    "c4b_ragged": lambda: wl.c4_bias_relu_chansum_backward(n=3, c=5, h=13, w=17),
    # a plan in stages: statistics over the outer axis in one sweep, the normalised tensor in a second
    "bn_ragged": lambda: wl.batch_norm_axis0(rows=1237, cols=77),
    "bn_f16": lambda: wl.batch_norm_axis0(rows=5000, cols=264, storage="f16"),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_config_parity(case, oracle, H):
    w = CASES[case]()
    print(f"[case] {case} {w.name} elements={w.elements}", flush=True)
    expr, stats = H.check_workload(w, oracle)
    print(f"[ok] {case} {expr.info()['kernel_class']} {stats}", flush=True)


# The sizes and launch configurations bench.py times.  The oracle (C, one thread per core) still
# finishes each of these in seconds, so every element is compared, not a sample.
FULL = {
    "c3_full": lambda: wl.c3_softmax_xent(),
    "c4_full": lambda: wl.c4_bias_relu_chansum(),
    "c5a_full": lambda: wl.c5_stress(reading="A"),
    "c5b_full": lambda: wl.c5_stress(reading="B"),
    "c3b_full": lambda: wl.c3_softmax_xent_backward(),
    "c4b_full": lambda: wl.c4_bias_relu_chansum_backward(),
    "bn_full": lambda: wl.batch_norm_axis0(),
}


@pytest.mark.parametrize("case", sorted(FULL))
def test_full_size_parity(case, oracle, H):
    import gc
    import torch
    w = FULL[case]()
    print(f"[case] {case} {w.name} elements={w.elements}", flush=True)
    expr, stats = H.check_workload(w, oracle, nthreads=16)
    print(f"[ok] {case} {expr.info()} {stats}", flush=True)
    del w, expr
    gc.collect()
    torch.cuda.empty_cache()


# Rows split over workgroups with a reduction over the rows to follow (the mean of the per-row
# losses): one stage of two launches -- the kernel that folds the rows' partials also folds the
# rows.  Many rows: a thread of that kernel per row; few, long rows: a wavefront per row.  Rows
# that hold NaN or infinities take the element-by-element rules inside the streaming kernel.
@pytest.mark.parametrize("rows,vocab,opts,per_thread", [
    (600, 40000, {"split_rows": 1}, True), (512, 131072, {}, True), (3, 1 << 20, {}, False), (37, 1003, {"split_rows": 1}, True),
    (70, 300000, {}, False), (600, 40000, {"split_rows": 1, "plain_extremes": 1}, True),
])
def test_split_rows_fold_the_mean_in_the_finish_kernel(rows, vocab, opts, per_thread, oracle, H):
    import gc
    import torch
    w = wl.c3_softmax_xent(rows=rows, vocab=vocab)
    x = w.buffers[0]
    inf = np.float32(np.inf)
    if rows >= 37:
        x[1, 5] = -inf; x[1, vocab - 3] = -inf
        x[2, :] = -inf
        x[3, 0] = -inf; x[3, 1] = 2.0
        x[4, 77] = inf
        x[5, vocab // 2] = np.nan; x[5, vocab // 2 + 9] = np.nan
        x[6, :] = 1.5
        x[7, vocab - 1] = 80.0
        x[8, 3] = 50.0; x[8, vocab - 2] = 50.0          # the maximum twice: the first index counts
    print(f"[case] split xent rows={rows} vocab={vocab} {opts}", flush=True)
    expr, got = H.run_gpu(w, **opts)
    info = expr.info()
    assert info["kernel_class"] == "multi" and info["grid_blocks"] == 1, info
    src = expr.source(0)
    assert "totx = AccX_combine()(totx, ax);" in src
    assert ("group = threadIdx.x" in src) == per_thread
    assert ("__builtin_fmaxf(vm_, xs" in src) == (not opts.get("plain_extremes"))
    want = oracle.evaluate(w.spec, wl.host_inputs(w), w.scalars, nthreads=16)
    for name, g, o, (rtol, atol) in zip(w.out_names, got, want, w.tol):
        H.compare(f"{name}", g, o, rtol, atol)
    del w, expr, got
    gc.collect()
    torch.cuda.empty_cache()


# Tuning options change how a kernel is generated and launched, never what it computes: every
# workload under every option still has to match the oracle.
OPTION_SETS = [
    {"force_scalar": 1}, {"force_index64": 1}, {"no_lds_staging": 1}, {"no_prefetch": 1}, {"no_prefetch": 2},
    {"xcd_remap": 1}, {"streaming": 1}, {"streaming": 2}, {"unroll": 1}, {"unroll": 4}, {"block_threads": 64},
    {"block_threads": 1024}, {"tile_elems": 1024}, {"waves_per_simd": 2}, {"max_blocks": 3}, {"no_rewrite": 1},
    {"split_rows": 1}, {"split_rows": 2}, {"plain_extremes": 1}, {"split_rows": 1, "plain_extremes": 1},
]
OPTION_CASES = ["c1_ragged", "c2_ragged", "c3_ragged", "c4_ragged", "c4_small", "c5a_small", "c5b_ragged_c", "c2b_ragged",
                "c3b_ragged", "c4b_ragged", "bn_ragged"]


@pytest.mark.parametrize("case", OPTION_CASES)
def test_options_do_not_change_results(case, oracle, H):
    from paper_1605_02688_amd import ewf
    w = CASES[case]()
    want = oracle.evaluate(w.oracle_spec or w.spec, wl.host_inputs(w), w.scalars, nthreads=8)
    ran = 0
    for opts in OPTION_SETS:
        print(f"[case] {case} {opts}", flush=True)
        try:
            expr, got = H.run_gpu(w, **opts)
        except ewf.EwfError as e:
            # an option that does not fit the workload is refused cleanly, never run wrongly
            assert e.status in (ewf.EUNSUPPORTED, ewf.EINVAL), (opts, e)
            print(f"[refused] {opts}: {e.message[:100]}", flush=True)
            continue
        for name, g, o, (rtol, atol) in zip(w.out_names, got, want, w.tol):
            H.compare(f"{w.name}.{name} {opts}", g, o, rtol, atol)
        ran += 1
    assert ran >= len(OPTION_SETS) - 3


# Partial results are folded in a fixed order by a second kernel (no atomics), so a workload gives
# the same bits on every run, whatever the workspace held before.
@pytest.mark.parametrize("case", ["c3_rows64", "c4_small", "c2b_full", "c3b_rows64", "c4b_small"])
def test_reductions_are_bitwise_reproducible(case, H):
    import torch
    from paper_1605_02688_amd import ewf
    w = CASES[case]()
    expr = ewf.Expression(w.spec)
    _bufs, ins = H.device_inputs(w)
    runs = []
    for fill in (0, -1, 0x7fc00000):
        outs = H.alloc_outputs(expr, w.spec, ins)
        nbytes = expr.plan(ins, outs)
        ws = torch.full((max(nbytes, 4) // 4 + 1,), fill, dtype=torch.int32, device="cuda") if nbytes else None
        expr.run(ins, outs, w.scalars, ws, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        runs.append([o.cpu().numpy().view(np.uint8 if o.element_size() == 1 else (np.uint16 if o.element_size() == 2 else np.uint32)) for o in outs])
    for other in runs[1:]:
        for a, b in zip(runs[0], other):
            assert np.array_equal(a, b)
