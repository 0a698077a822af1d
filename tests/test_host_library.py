"""Host-only tests of the library: the C ABI surface, graph validation, the stride /
broadcast canonicaliser, kernel-class selection and run-time code generation (the run-time
compiler cross-compiles for gfx950 without a GPU).  No kernel is launched here."""
import os
import re

import numpy as np
import pytest

from paper_1605_02688_amd import ewf
from paper_1605_02688_amd.selfcheck import plan_layout
from workloads import GraphSpec
from workloads import configs as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
BASE = 0x7F0000000000


def contig(shape):
    st, acc = [], 1
    for e in reversed(shape):
        st.append(acc)
        acc *= e
    return tuple(reversed(st))


def ref(addr, shape, strides=None):
    return ewf.TensorRef(addr, tuple(shape), tuple(strides) if strides is not None else contig(shape))


def plan_workload(w, **opts):
    expr = ewf.Expression(w.spec, **opts)
    ws, info = plan_layout(expr, w.spec, w.views, [w.buffers[v.buffer].itemsize for v in w.views])
    return expr, ws, info


def strides_of(expr, info):
    return [ewf.debug_operand_strides(expr.handle, k, info["rank"]) for k in range(info["noperands"])]


# ------------------------------------------------------------------ ABI surface

def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "ewf.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(ewf_[a-z0-9_]+)\s*\(", header))
    assert len(declared) >= 20
    import ctypes
    lib = ctypes.CDLL(ewf.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), f"{name} declared in ewf.h but not exported"
    assert declared == set(ewf.EXPORTED)


def test_error_message_is_thread_local_text():
    with pytest.raises(ewf.EwfError) as e:
        ewf.graph_create(99)
    assert e.value.status == ewf.EINVAL and "rank" in e.value.message


# ------------------------------------------------------------------ graph validation

def test_type_rules():
    g = ewf.graph_create(1)
    f = ewf.input(g, ewf.F32, [0]); i = ewf.input(g, ewf.I32, [0]); h = ewf.input(g, ewf.F16, [0])
    with pytest.raises(ewf.EwfError) as e:
        ewf.apply(g, ewf.OPS["add"], [f, i])
    assert e.value.status == ewf.ETYPE
    with pytest.raises(ewf.EwfError) as e:
        ewf.apply(g, ewf.OPS["exp"], [i])
    assert e.value.status == ewf.ETYPE
    with pytest.raises(ewf.EwfError) as e:
        ewf.apply(g, ewf.OPS["add"], [f])
    assert e.value.status == ewf.EINVAL
    with pytest.raises(ewf.EwfError) as e:
        ewf.apply(g, ewf.OPS["add"], [f, 77])
    assert e.value.status == ewf.EINVAL
    assert ewf.apply(g, ewf.OPS["add"], [f, h]) >= 0            # f16 storage is an f32 value
    c = ewf.apply(g, ewf.OPS["gt"], [f, h])
    with pytest.raises(ewf.EwfError) as e:
        ewf.output(g, c, ewf.F32)                                 # comparison results are int32
    assert e.value.status == ewf.ETYPE
    ewf.output(g, c, ewf.I32)
    ewf.output(g, ewf.cast(g, c, ewf.F32), ewf.F16)
    with pytest.raises(ewf.EwfError):
        ewf.scalar(g, ewf.F16)
    with pytest.raises(ewf.EwfError):
        ewf.iota(g, 1)
    with pytest.raises(ewf.EwfError) as e:
        ewf.reduce(g, ewf.REDOPS["sum"], f, [1], False)
    assert e.value.status == ewf.EINVAL
    with pytest.raises(ewf.EwfError):
        ewf.reduce(g, ewf.REDOPS["sum"], f, [0, 0], False)
    ewf.graph_destroy(g)
    g = ewf.graph_create(2)
    x = ewf.input(g, ewf.F32, [0, 0])
    am = ewf.reduce(g, ewf.REDOPS["argmax"], x, [0, 1], False)    # arg-max over several axes: an int32 position
    assert am >= 0
    with pytest.raises(ewf.EwfError) as e:
        ewf.compile(g)                                            # no output declared
    assert e.value.status == ewf.EINVAL
    ewf.graph_destroy(g)


def test_output_shapes_follow_keep_flag():
    w = wl.layout_only(wl.c3_softmax_xent, rows=12, vocab=30)
    expr = ewf.Expression(w.spec)
    ins = [ref(BASE, (12, 30)), ref(BASE + (1 << 20), (12, 1))]
    assert expr.output_shapes(ins) == [(12,), (12,), (12,), (12,), (), (12,)]
    s = GraphSpec(3)
    x = s.input("f32", (False, False, False))
    r = s.reduce("sum", x, (0, 2), keep=True)
    s.output(r, "f32")
    s.output(s.mul(r, s.reduce("max", x, (2,), keep=False)), "f32")
    expr = ewf.Expression(s)
    # an axis dropped by any operand stays dropped where the result is broadcastable
    assert expr.output_shapes([ref(BASE, (4, 5, 6))]) == [(1, 5, 1), (4, 5)]


# ------------------------------------------------------------------ canonical forms of the workloads

def test_c1_canonical_form():
    expr, ws, info = plan_workload(wl.layout_only(wl.c1_affine_tanh))
    assert info["kernel_class"] == "tile" and ws == 0
    assert info["rank"] == 2 and info["extent"] == (1024, 256)       # b [1,256] blocks the merge
    assert info["vec"] == 4 and info["index_bits"] == 32
    assert strides_of(expr, info) == [(256, 1), (0, 1), (256, 1)]


def test_c2_canonical_form():
    expr, ws, info = plan_workload(wl.layout_only(wl.c2_lstm_cell))
    assert info["kernel_class"] == "tile" and info["extent"] == (64, 1024) and info["vec"] == 4
    st = strides_of(expr, info)
    assert st[:4] == [(4096, 1)] * 4 and st[4:8] == [(0, 1)] * 4 and st[8:] == [(1024, 1)] * 3


def test_c3_canonical_form():
    expr, ws, info = plan_workload(wl.layout_only(wl.c3_softmax_xent))
    assert info["kernel_class"] == "row" and info["extent"] == (1280, 10000)
    assert info["reduced"] == (False, True) and info["vec"] == 4
    st = strides_of(expr, info)
    assert st[0] == (10000, 1) and st[1] == (1, 0)
    assert ws == 1280 * 4                                            # one loss value per row


def test_c4_canonical_form():
    expr, ws, info = plan_workload(wl.layout_only(wl.c4_bias_relu_chansum))
    assert info["kernel_class"] == "tile_reduce"
    assert info["extent"] == (128, 64, 12544) and info["reduced"] == (True, False, True)
    st = strides_of(expr, info)
    assert st[0] == (802816, 12544, 1) and st[1] == (0, 1, 0) and st[2] == (0, 1, 0)
    assert st[3] == (802816, 12544, 1) and st[4] == (0, 1, 0)
    assert info["tile"][0] == 1 and info["tile"][1] == 1              # a tile never leaves its channel


@pytest.mark.parametrize("reading,x3", [("A", (802816, 1, 14336, 256)), ("B", (802816, 56, 1, 14336))])
def test_c5_canonical_form(reading, x3):
    expr, ws, info = plan_workload(wl.layout_only(wl.c5_stress, reading=reading), no_lds_staging=1)
    assert info["kernel_class"] == "tile" and info["extent"] == (64, 256, 56, 56)   # nothing merges
    assert info["vec"] == 8 and info["index_bits"] == 32
    st = strides_of(expr, info)
    assert st[0] == st[1] == st[2] == st[6] == (802816, 3136, 56, 1)
    assert st[3] == x3 and st[4] == (0, 56, 0, 1) and st[5] == (0, 56, 1, 0)


def test_contiguous_operands_collapse_to_one_dimension():
    s = GraphSpec(4)
    s.output(s.apply("exp", s.add(s.input("f32", (False,) * 4), s.input("f32", (False,) * 4))), "f32")
    expr = ewf.Expression(s)
    shape = (6, 5, 4, 8)
    expr.plan([ref(BASE, shape), ref(BASE + (1 << 24), shape)], [ref(BASE + (2 << 24), shape)])
    info = expr.info()
    assert info["rank"] == 1 and info["extent"] == (960,) and info["vec"] == 4
    # a transposed input keeps two dimensions; the output's memory order leads
    expr.plan([ref(BASE, (6, 5, 4, 8)), ref(BASE + (1 << 24), shape, (160, 8, 40, 1))], [ref(BASE + (2 << 24), shape)])
    info = expr.info()
    assert info["extent"] == (6, 5, 4, 8)[0:1] + (5, 4, 8) or info["rank"] >= 3


def test_extent_one_dimensions_disappear_and_single_element():
    s = GraphSpec(3)
    s.output(s.apply("tanh", s.input("f32", (False, False, False))), "f32")
    expr = ewf.Expression(s)
    expr.plan([ref(BASE, (1, 7, 1))], [ref(BASE + 4096, (1, 7, 1))])
    assert expr.info()["extent"] == (7,)
    expr.plan([ref(BASE, (1, 1, 1))], [ref(BASE + 4096, (1, 1, 1))])
    assert expr.info()["extent"] == (1,) and expr.info()["grid_blocks"] == 1


def test_vector_width_follows_alignment_and_extent():
    s = GraphSpec(2)
    s.output(s.apply("neg", s.input("f32", (False, False))), "f32")
    expr = ewf.Expression(s)
    expr.plan([ref(BASE, (8, 64))], [ref(BASE + (1 << 20), (8, 64))])
    assert expr.info()["vec"] == 4
    expr.plan([ref(BASE + 8, (8, 64))], [ref(BASE + (1 << 20), (8, 64))])       # 8-byte aligned input
    assert expr.info()["vec"] == 2
    expr.plan([ref(BASE + 4, (8, 64))], [ref(BASE + (1 << 20), (8, 64))])
    assert expr.info()["vec"] == 1
    expr.plan([ref(BASE, (8, 63), (64, 1))], [ref(BASE + (1 << 20), (8, 63), (64, 1))])  # odd row length
    assert expr.info()["vec"] == 1
    expr.plan([ref(BASE, (8, 62), (66, 1))], [ref(BASE + (1 << 20), (8, 62), (66, 1))])  # rows 8-byte aligned
    assert expr.info()["vec"] == 2
    e2 = ewf.Expression(s, force_scalar=1)
    e2.plan([ref(BASE, (8, 64))], [ref(BASE + (1 << 20), (8, 64))])
    assert e2.info()["vec"] == 1


def test_wide_accesses_where_only_the_element_is_aligned():
    """Reducing tile kernels, and element-wise ones on 2-byte storage, keep the full vector width on
    rows of odd pitch or length: accesses that assume element alignment, the vector that a row's
    end cuts element by element.  Other classes and float32 element-wise kernels stay strict."""
    s = GraphSpec(2)
    x = s.input("f32", (False, False))
    s.output(s.reduce("sum", x, (1,)), "f32"); s.output(s.reduce("max", x, (1,)), "f32")
    e = ewf.Expression(s)
    e.plan([ref(BASE, (40, 50257))], [ref(BASE + (1 << 30), (40,)), ref(BASE + (1 << 31), (40,))])
    assert e.info()["kernel_class"] == "tile_reduce" and e.info()["vec"] == 4
    src = e.source()
    assert "ewf_ld_u<float, EWF_VEC>" in src and "it.nv[u]" in src and e.info()["tile"][1] % 4 == 0
    # an even length behind an odd starting element: no vector is cut
    e.plan([ref(BASE + 4, (40, 50256), (50260, 1))], [ref(BASE + (1 << 30), (40,)), ref(BASE + (1 << 31), (40,))])
    assert e.info()["vec"] == 4 and "ewf_ld_u<" in e.source() and "it.nv" not in e.source()
    # aligned rows: the ordinary accesses
    e.plan([ref(BASE, (40, 50256))], [ref(BASE + (1 << 30), (40,)), ref(BASE + (1 << 31), (40,))])
    assert e.info()["vec"] == 4 and "ewf_ld_u<" not in e.source()
    assert ewf.Expression(s, force_scalar=1).plan([ref(BASE, (40, 50257))], [ref(BASE + (1 << 30), (40,)), ref(BASE + (1 << 31), (40,))]) >= 0
    # the row class does the same for rows it holds in registers
    e3 = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=1280, vocab=10001))[0]
    assert e3.info()["kernel_class"] == "row" and e3.info()["vec"] == 4 and e3.info()["block_threads"] == 256
    assert "ewf_ld_u<float, EWF_VEC>" in e3.source() and "col + e_ >= cols" in e3.source()
    # a plan that is generated more than once (another block size after the first attempt) keeps
    # the accesses that go with its width
    e4 = plan_workload(wl.layout_only(wl.c3_softmax_xent_backward, rows=300, vocab=20003))[0]
    assert e4.info()["kernel_class"] == "row" and e4.info()["vec"] == 4 and e4.info()["block_threads"] == 512
    assert "ewf_ld_u<float, EWF_VEC>" in e4.source() and "ewf_ld<float, EWF_VEC>" not in e4.source() and "ewf_st_u<float, EWF_VEC>" in e4.source()
    # element-wise: float16 yes, float32 no
    for dt, vec in (("f16", 8), ("f32", 1)):
        s2 = GraphSpec(1)
        s2.output(s2.apply("tanh", s2.input(dt, (False,))), dt)
        e2 = ewf.Expression(s2)
        e2.plan([ref(BASE, ((1 << 22) + 3,))], [ref(BASE + (1 << 30), ((1 << 22) + 3,))])
        assert e2.info()["vec"] == vec and ("ewf_st_u<" in e2.source()) == (dt == "f16"), (dt, e2.info())


def test_index_width_selection():
    s = GraphSpec(2)
    s.output(s.apply("neg", s.input("f16", (False, False))), "f16")
    expr = ewf.Expression(s)
    expr.plan([ref(BASE, (1 << 15, 1 << 15))], [ref(BASE + (1 << 40), (1 << 15, 1 << 15))])
    assert expr.info()["index_bits"] == 32                         # 2^30 elements
    expr.plan([ref(BASE, (1 << 16, 1 << 15))], [ref(BASE + (1 << 40), (1 << 16, 1 << 15))])
    assert expr.info()["index_bits"] == 64                         # 2^31 elements
    # few elements but a huge stride also needs 64-bit offsets
    expr.plan([ref(BASE, (4, 16), (1 << 31, 1))], [ref(BASE + (1 << 40), (4, 16))])
    assert expr.info()["index_bits"] == 64
    e2 = ewf.Expression(s, force_index64=1)
    e2.plan([ref(BASE, (4, 16))], [ref(BASE + (1 << 40), (4, 16))])
    assert e2.info()["index_bits"] == 64 and "long long idx_t" in e2.source()


def test_long_or_few_rows_are_split_over_workgroups():
    # softmax cross-entropy: one workgroup per row while a row sits well in registers ...
    def plan(rows, vocab, maker=wl.c3_softmax_xent, **opts):
        w = wl.layout_only(maker, rows=rows, vocab=vocab)
        return plan_workload(w, **opts)[0]
    assert plan(1280, 10000).info()["kernel_class"] == "row"
    assert plan(2048, 24000).info()["kernel_class"] == "row"
    # ... otherwise the chain max -> sum of exp(x - max) becomes one reduction level whose
    # (maximum, sum) pair is rescaled as the maximum grows, and rows are split over workgroups
    for rows, vocab in ((1024, 65536), (640, 100000), (64, 1 << 20), (100, 20000), (2048, 32768)):
        e = plan(rows, vocab)
        info = e.info()
        assert info["kernel_class"] == "multi" and info["grid_blocks"] == 1, (rows, vocab, info)
        first = e.info(0)
        assert first["kernel_class"] == "tile_reduce" and first["extent"] == (rows, vocab)
        src = e.source(0)
        assert "* w_ + 1.0f" in src and "ewf_fast::exp(-__builtin_fabsf(d_))" in src
        assert "__builtin_fmaxf(vm_, xs" in src                          # finite vectors are folded whole
        assert len(re.findall(r"ewf_ld(?:_nt)?<float, EWF_VEC>", src)) == 1      # the logits are read once
        # the mean over the per-row losses is folded by the same kernel that folds the rows' partials
        assert "totx = AccX_combine()(totx, ax);" in src and src.count("__global__") == 2
    # the caller can insist either way
    assert plan(640, 100000, split_rows=2).info()["kernel_class"] == "row"
    assert plan(1280, 10000, split_rows=1).info()["kernel_class"] == "multi"
    # backward: the statistics in one pass, the gradient in a second
    e = plan(512, 131072, maker=wl.c3_softmax_xent_backward)
    assert e.info()["kernel_class"] == "multi" and [e.info(k)["kernel_class"] for k in range(2)] == ["tile_reduce", "tile"]
    # plain row reductions never needed the row class
    s = GraphSpec(2)
    s.output(s.reduce("sum", s.input("f32", (False, False)), (1,)), "f32")
    e = ewf.Expression(s, split_rows=1)
    e.plan([ref(BASE, (1000, 4096))], [ref(BASE + (1 << 30), (1000,))])
    assert e.info()["kernel_class"] == "tile_reduce"


def test_an_input_that_a_later_stage_reads_again_is_left_in_the_cache():
    # batch normalisation over axis 0: statistics in one kernel, the normalised tensor in a second.
    # The first kernel loads X with ordinary accesses; the second one, its last reader, streams
    # it.  (Measured up to a gigabyte; beyond that both stream.)
    def sources(rows, **opts):
        e, _, info = plan_workload(wl.layout_only(wl.batch_norm_axis0, rows=rows, cols=1024), **opts)
        assert info["kernel_class"] == "multi" and info["grid_blocks"] == 2
        return e.source(0), e.source(1)
    first, second = sources(32768)                       # 134 MB
    assert "ewf_ld<float, EWF_VEC>" in first and "ewf_ld_nt<float, EWF_VEC>" not in first
    assert "ewf_ld_nt<float, EWF_VEC>" in second and "ewf_st_nt<float, EWF_VEC>" in second
    first, second = sources(65536)                       # 268 MB: more than the cache holds, part of it survives
    assert "ewf_ld_nt<float, EWF_VEC>" not in first and "ewf_ld_nt<float, EWF_VEC>" in second
    first, second = sources(524288)                      # 2.1 GB
    assert "ewf_ld_nt<float, EWF_VEC>" in first and "ewf_ld_nt<float, EWF_VEC>" in second
    first, _ = sources(32768, streaming=1)               # the caller's choice stands
    assert "ewf_ld_nt<float, EWF_VEC>" in first


def test_argmax_positions_must_fit_int32():
    s = GraphSpec(2)
    s.output(s.reduce("argmax", s.input("f16", (False, False)), (0, 1)), "i32")
    e = ewf.Expression(s)
    with pytest.raises(ewf.EwfError) as err:
        e.plan([ref(BASE, (70000, 40000))], [ref(BASE + (1 << 40), ())])
    assert err.value.status == ewf.ESHAPE and "int32" in err.value.message
    e.plan([ref(BASE, (7000, 40000))], [ref(BASE + (1 << 40), ())])          # 2.8e8 positions: fine
    src = e.source() or e.source(0)
    assert "p.ext[" in src and "i0" in src


def test_chains_that_passes_cannot_shorten_stay_with_the_row_class():
    # layer normalisation: mean, then the variance of the centred values, then an output that uses
    # both and two more rows (scale, shift).  A plan in passes would sweep the tensor three times.
    def plan(rows, cols, dt, **opts):
        s = GraphSpec(2)
        x = s.input(dt, (False, False)); ga = s.input("f32", (True, False)); be = s.input("f32", (True, False))
        mean = s.mul(s.reduce("sum", x, (1,), keep=True), s.const(1.0 / cols))
        xc = s.sub(x, mean)
        var = s.mul(s.reduce("sum", s.mul(xc, xc), (1,), keep=True), s.const(1.0 / cols))
        s.output(s.add(s.mul(s.mul(xc, s.apply("recip", s.apply("sqrt", s.add(var, s.const(1e-5))))), ga), be), dt)
        e = ewf.Expression(s, **opts)
        e.plan([ref(BASE, (rows, cols)), ref(BASE + (1 << 34), (1, cols)), ref(BASE + (1 << 35), (1, cols))], [ref(BASE + (1 << 36), (rows, cols))])
        return e
    for rows, cols, dt in ((4096, 16384, "f32"), (4096, 16384, "f16"), (1024, 65536, "f16"), (8192, 8192, "f32")):
        e = plan(rows, cols, dt)
        assert e.info()["kernel_class"] == "row", (rows, cols, dt, e.info())
        src = e.source()
        # the row itself is held in registers; scale and shift are read where the output is written
        assert "x_in0[" in src and "x_in1[" not in src and "w_in1" in src and "w_in2" in src
    assert plan(4096, 16384, "f32", split_rows=1).info()["kernel_class"] == "multi"
    assert plan(50000, 512, "f32").info()["kernel_class"] == "lane"


def test_short_rows_share_a_wavefront():
    # softmax cross-entropy over 8 classes (32-byte rows): one thread per row when there are many rows
    e = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=50000, vocab=8))[0]
    assert e.info()["kernel_class"] == "lane" and e.info()["grid_blocks"] == (50000 + 255) // 256
    assert "ewf_lane_xor" not in e.source() and "ewf_block_reduce" in e.source()      # no lane exchange; the mean is folded by the second kernel
    # 12 classes: four lanes per row (the fourth has no column), two butterfly steps
    e = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=50000, vocab=12))[0]
    assert e.info()["kernel_class"] == "lane" and e.info()["grid_blocks"] == (50000 + 63) // 64       # fewer than the resident grid's cap
    assert e.source().count("ewf_lane_xor(acc1, ") == 2
    # rows of 100 float32: 32 lanes per row, five butterfly steps per reduction level
    e = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=50000, vocab=100))[0]
    assert e.info()["kernel_class"] == "lane" and e.info()["grid_blocks"] == 2048                     # a resident grid strides over the rows
    assert e.source().count("ewf_lane_xor(acc1, ") == 5 and "ewf_lane_xor(acc1, 16)" in e.source()
    # few rows, or longer ones: a wavefront or more per row
    assert plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=1000, vocab=12))[0].info()["kernel_class"] == "row"
    assert plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=50000, vocab=2048))[0].info()["kernel_class"] == "row"
    # rows of up to 4096 bytes: a wavefront per row, several vectors per lane, four rows per workgroup
    e = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=50000, vocab=512))[0]
    assert e.info()["kernel_class"] == "lane" and e.info()["block_threads"] == 256 and "ewf_lane_xor(acc1, 32)" in e.source()
    # more rows than one workgroup should fold: the mean becomes a pass of its own
    e = plan_workload(wl.layout_only(wl.c3_softmax_xent, rows=200000, vocab=12))[0]
    assert e.info()["kernel_class"] == "multi" and e.info(0)["kernel_class"] == "lane"


# ------------------------------------------------------------------ shape / alias / argument errors

def _add2():
    s = GraphSpec(2)
    s.output(s.add(s.input("f32", (False, False)), s.input("f32", (True, False))), "f32")
    return ewf.Expression(s)


def test_broadcast_pattern_is_enforced():
    expr = _add2()
    out = ref(BASE + (2 << 20), (3, 4))
    expr.plan([ref(BASE, (3, 4)), ref(BASE + (1 << 20), (1, 4))], [out])
    with pytest.raises(ewf.EwfError) as e:                           # flagged dimension with extent 3
        expr.plan([ref(BASE, (3, 4)), ref(BASE + (1 << 20), (3, 4))], [out])
    assert e.value.status == ewf.ESHAPE
    with pytest.raises(ewf.EwfError) as e:                           # unflagged extent 1 never broadcasts
        expr.plan([ref(BASE, (1, 4)), ref(BASE + (1 << 20), (1, 4))], [out])
    assert e.value.status == ewf.ESHAPE
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(BASE, (3, 4)), ref(BASE + (1 << 20), (1, 5))], [out])
    assert e.value.status == ewf.ESHAPE
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(BASE, (3, 4)), ref(BASE + (1 << 20), (1, 4))], [ref(BASE + (2 << 20), (4, 3))])
    assert e.value.status == ewf.ESHAPE
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(BASE, (3, 4))], [out])
    assert e.value.status == ewf.EINVAL
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(BASE, (3, 4), (4, -1)), ref(BASE + (1 << 20), (1, 4))], [out])
    assert e.value.status == ewf.EINVAL
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(0, (3, 4)), ref(BASE + (1 << 20), (1, 4))], [out])
    assert e.value.status == ewf.EINVAL


def test_aliasing_rules():
    expr = _add2()
    a = ref(BASE, (8, 16)); b = ref(BASE + (1 << 20), (1, 16))
    expr.plan([a, b], [ref(BASE, (8, 16))])                            # exact alias: in place
    with pytest.raises(ewf.EwfError) as e:                             # shifted by one row
        expr.plan([a, b], [ref(BASE + 64, (8, 16))])
    assert e.value.status == ewf.EALIAS
    with pytest.raises(ewf.EwfError) as e:                             # same memory, transposed walk
        expr.plan([ref(BASE, (16, 16)), ref(BASE + (1 << 20), (1, 16))], [ref(BASE, (16, 16), (1, 16))])
    assert e.value.status == ewf.EALIAS
    with pytest.raises(ewf.EwfError) as e:                             # output that writes an element twice
        expr.plan([a, b], [ref(BASE + (2 << 20), (8, 16), (0, 1))])
    assert e.value.status == ewf.EALIAS
    # column blocks of one buffer interleave in address range but share no element
    expr.plan([ref(BASE, (8, 16), (64, 1)), b], [ref(BASE + 16 * 4, (8, 16), (64, 1))])
    with pytest.raises(ewf.EwfError) as e:
        expr.plan([ref(BASE, (8, 16), (64, 1)), b], [ref(BASE + 8 * 4, (8, 16), (64, 1))])
    assert e.value.status == ewf.EALIAS
    # two outputs must not share elements either
    s = GraphSpec(1)
    x = s.input("f32", (False,))
    s.output(s.apply("exp", x), "f32"); s.output(s.apply("neg", x), "f32")
    e2 = ewf.Expression(s)
    with pytest.raises(ewf.EwfError) as e:
        e2.plan([ref(BASE, (64,))], [ref(BASE + 4096, (64,)), ref(BASE + 4096 + 128, (64,))])
    assert e.value.status == ewf.EALIAS
    e2.plan([ref(BASE, (64,))], [ref(BASE + 4096, (64,)), ref(BASE + 8192, (64,))])


def test_zero_size_is_success_without_kernel():
    expr = _add2()
    ws = expr.plan([ref(0, (0, 4)), ref(BASE, (1, 4))], [ref(0, (0, 4))])
    assert ws == 0 and expr.info()["kernel_class"] == "none"
    s = GraphSpec(2)
    s.output(s.reduce("max", s.input("f32", (False, False)), (1,)), "f32")
    with pytest.raises(ewf.EwfError) as e:
        ewf.Expression(s).plan([ref(BASE, (3, 0))], [ref(BASE + 4096, (3,))])
    assert e.value.status == ewf.ESHAPE
    # a sum or a product over an empty axis has an identity: planned (a fill at run time)
    for red_ in ("sum", "prod"):
        s = GraphSpec(2)
        s.output(s.reduce(red_, s.input("f32", (False, False)), (1,)), "f32")
        e3 = ewf.Expression(s)
        assert e3.plan([ref(BASE, (3, 0))], [ref(BASE + 4096, (3,))]) == 0 and e3.info()["kernel_class"] == "none"
    # a value computed from such a reduction: the reduction becomes a temporary holding the identity
    # and one kernel computes the value from it
    s = GraphSpec(2)
    s.output(s.apply("exp", s.reduce("sum", s.input("f32", (False, False)), (1,))), "f32")
    e4 = ewf.Expression(s)
    assert e4.plan([ref(BASE, (3, 0))], [ref(BASE + 4096, (3,))]) >= 12
    assert e4.info()["kernel_class"] == "multi" and e4.info()["grid_blocks"] == 1 and e4.info(0)["kernel_class"] == "tile"
    s = GraphSpec(2)
    s.output(s.apply("exp", s.reduce("max", s.input("f32", (False, False)), (1,))), "f32")
    with pytest.raises(ewf.EwfError) as e:
        ewf.Expression(s).plan([ref(BASE, (3, 0))], [ref(BASE + 4096, (3,))])
    assert e.value.status == ewf.ESHAPE


# ------------------------------------------------------------------ kernel classes and code generation

def test_kernel_class_selection():
    def red(ndim, axes, shape, strides=None, extra=None):
        s = GraphSpec(ndim)
        x = s.input("f32", (False,) * ndim)
        r = s.reduce("sum", x, axes)
        s.output(r, "f32")
        if extra:
            extra(s, x, r)
        expr = ewf.Expression(s)
        ins = [ref(BASE, shape, strides)]
        outs = [ref(BASE + (1 << 36) + k * (1 << 32), sh) for k, sh in enumerate(expr.output_shapes(ins))]
        expr.plan(ins, outs)
        return expr.info()
    assert red(2, (1,), (4096, 512))["kernel_class"] == "lane"           # many short rows: a wavefront each
    assert red(2, (1,), (4096, 2048))["kernel_class"] == "row"           # longer ones: a workgroup each
    assert red(2, (1,), (4, 1 << 20))["kernel_class"] == "tile_reduce"    # few long rows: split them
    assert red(1, (0,), (1 << 20,))["kernel_class"] == "tile_reduce"      # full reduction
    assert red(3, (0, 2), (8, 16, 256))["kernel_class"] == "tile_reduce"
    assert red(3, (1, 2), (64, 8, 32))["extent"] == (64, 256)            # reduced axes merge
    # softmax: the output depends on a reduction and varies along the row -> row-resident class
    info = red(2, (1,), (4, 1000), extra=lambda s, x, r: s.output(s.div(x, r), "f32"))
    assert info["kernel_class"] == "row"
    # the kept axis is the fastest-varying one: column class, lanes along the columns
    info = red(2, (0,), (512, 512))
    assert info["kernel_class"] == "col" and info["reduced"] == (True, False)
    assert red(4, (0, 2), (6, 50, 7, 32))["kernel_class"] == "col"
    assert red(2, (1,), (200, 96), strides=(1, 200))["kernel_class"] == "col"   # a transposed view, reduced along its rows
    # normalising by a column sum needs a second pass over memory: two stages
    info = red(2, (0,), (512, 512), extra=lambda s, x, r: s.output(s.div(x, r), "f32"))
    assert info["kernel_class"] == "multi" and info["grid_blocks"] == 2
    # reducing over extent-1 axes is the identity: plain element-wise kernel
    assert red(2, (1,), (64, 1))["kernel_class"] == "tile"


def test_generated_source_structure_and_cache():
    w = wl.layout_only(wl.c1_affine_tanh, rows=8192)
    w.spec.nodes.append(("const", "f32", 0.12345678))       # makes this source unique in the process-wide cache
    expr, _, info = plan_workload(w)
    src = expr.source()
    assert "ewf_kernel" in src and "ewf_fast::tanh" in src and "ewf_ld<float, EWF_VEC>" in src
    assert "p.s0" in src                                   # the run-time scalar is a kernel argument
    n0 = ewf.debug_compile_count(expr.handle)
    assert n0 <= 1
    # another number of rows: same layout class, same source, nothing recompiled
    w2 = wl.layout_only(wl.c1_affine_tanh, rows=16384)
    ws, info2 = plan_layout(expr, w2.spec, w2.views, [4, 4])
    assert expr.source() == src and ewf.debug_compile_count(expr.handle) == n0
    # a literal is baked into the code
    wc = wl.layout_only(wl.c1_affine_tanh, a_form="const")
    exprc, _, _ = plan_workload(wc)
    assert "0x3f000000" in exprc.source() and "p.s0" not in exprc.source()


def _values(expr):
    return [l.split("=", 1)[1].strip() for l in expr.source().split("\n")
            if l.strip().startswith(("const float v", "const int v"))]


def test_scalar_graph_rewrites():
    """Canonicalisation and stabilisation of the scalar graph (paper section 2.2.1): merged
    duplicates, folded constants, log(1+x) -> log1p(x), exp(x)-1 -> expm1(x), x*x and
    pow(x,2) -> a square, identities removed."""
    def planned(s, n=1024, **opts):
        expr = ewf.Expression(s, **opts)
        ins = [ref(BASE + k * (1 << 24), (n,)) for k in range(sum(1 for nd in s.nodes if nd[0] == "input"))]
        outs = [ref(BASE + (1 << 36) + k * (1 << 24), sh) for k, sh in enumerate(expr.output_shapes(ins))]
        expr.plan(ins, outs)
        return expr
    s = GraphSpec(1); x = s.input("f32", (False,))
    a = s.apply("log", s.add(s.const(1.0), s.apply("exp", x)))
    b = s.apply("log", s.add(s.apply("exp", x), s.const(1.0)))       # the same value, written the other way round
    c = s.sub(s.apply("exp", x), s.const(1.0))
    d = s.apply("pow", s.mul(x, s.const(1.0)), s.const(2.0))
    k = s.mul(s.const(2.0), s.const(3.0))
    s.output(s.add(s.add(a, b), s.mul(s.add(c, d), k)), "f32")
    expr = planned(s)
    before, after = expr.graph_size()
    assert before == 23 and after == 10
    vals = " ".join(_values(expr))
    assert vals.count("::exp(") == 1 and vals.count("::log1p(") == 1 and vals.count("::expm1(") == 1
    assert "::log(" not in vals and "::pow" not in vals and "0x40c00000u" in vals       # 2 * 3 folded to 6.0f
    raw = planned(s, no_rewrite=1)
    assert raw.graph_size() == (23, 23) and " ".join(_values(raw)).count("::exp(") == 3

    # integer folding wraps around; casts fold; comparisons fold to 0/1
    s = GraphSpec(1); i = s.input("i32", (False,))
    big = s.mul(s.const(65536, "i32"), s.const(65536, "i32"))                           # 2^32 wraps to 0
    one = s.apply("gt", s.const(2.5), s.const(1.0))
    s.output(s.add(s.add(i, big), s.add(one, s.cast(s.const(-3.9), "i32"))), "i32")   # i + 0 + (1 + -3)
    expr = planned(s)
    assert "0xfffffffeu" in " ".join(_values(expr)) and expr.graph_size()[1] == 3     # input, literal -2, add

    # a rewrite never changes an output's shape: where(true, row_vector, full) keeps the full extent
    s = GraphSpec(2)
    rowv = s.input("f32", (True, False)); fullv = s.input("f32", (False, False))
    s.output(s.apply("where", s.const(1, "i32"), rowv, fullv), "f32")
    expr = ewf.Expression(s)
    ins = [ref(BASE, (1, 64)), ref(BASE + (1 << 24), (8, 64))]
    assert expr.output_shapes(ins) == [(8, 64)]
    # ... while where(true, a, b) with equal patterns is just a
    s = GraphSpec(1); p_ = s.input("f32", (False,)); q_ = s.input("f32", (False,))
    s.output(s.apply("where", s.const(1, "i32"), s.apply("tanh", p_), s.apply("exp", q_)), "f32")
    expr = planned(s)
    assert "::exp(" not in " ".join(_values(expr)) and "::tanh(" in " ".join(_values(expr))

    # reductions merge too: two sums of the same argument over the same axes are one accumulator
    s = GraphSpec(2); x = s.input("f32", (False, False))
    e1 = s.apply("exp", x); e2 = s.apply("exp", x)
    s.output(s.reduce("sum", e1, (1,)), "f32"); s.output(s.reduce("sum", e2, (1,)), "f32")
    expr = ewf.Expression(s)
    ins = [ref(BASE, (600, 128))]
    outs = [ref(BASE + (1 << 36) + k * (1 << 24), sh) for k, sh in enumerate(expr.output_shapes(ins))]
    expr.plan(ins, outs)
    assert expr.graph_size() == (5, 3) and "float a1;" not in expr.source()


def test_disk_cache_of_compiled_kernels(tmp_path):
    """A second process finds the code object of the first on disk and compiles nothing (paper
    section 2.2.3: compiled modules are cached persistently)."""
    import json, subprocess, sys, os
    script = (
        "import sys, json; sys.path.insert(0, %r)\n"
        "from paper_1605_02688_amd import ewf\n"
        "from workloads import GraphSpec\n"
        "s = GraphSpec(1); x = s.input('f32', (False,))\n"
        "s.output(s.apply('tanh', s.mul(x, s.const(0.4242))), 'f32')\n"
        "e = ewf.Expression(s)\n"
        "B = 0x7F0000000000\n"
        "e.plan([ewf.TensorRef(B, (4096,), (1,))], [ewf.TensorRef(B + (1 << 20), (4096,), (1,))])\n"
        "print(json.dumps(ewf.debug_cache_stats()))\n" % ROOT)
    env = dict(os.environ, EWF_CACHE_DIR=str(tmp_path))
    runs = [json.loads(subprocess.run([sys.executable, "-c", script], env=env, capture_output=True, text=True, check=True).stdout.strip().split("\n")[-1])
            for _ in range(2)]
    assert runs[0] == {"memory_hits": 0, "disk_hits": 0, "compiles": 1}
    assert runs[1] == {"memory_hits": 0, "disk_hits": 1, "compiles": 0}
    files = [f for f in os.listdir(tmp_path) if f.endswith(".co")]
    assert len(files) == 1
    # a damaged file is ignored, not trusted
    with open(os.path.join(tmp_path, files[0]), "r+b") as f:
        f.seek(6); f.write(b"\x01\x02")
    again = json.loads(subprocess.run([sys.executable, "-c", script], env=env, capture_output=True, text=True, check=True).stdout.strip().split("\n")[-1])
    assert again["compiles"] == 1 and again["disk_hits"] == 0


def test_math_mode_follows_storage():
    w5 = wl.layout_only(wl.c5_stress, n=2)
    e5, _, _ = plan_workload(w5)
    assert "ewf_bare::exp" in e5.source() and "ewf_acc::" not in e5.source()     # float16 outputs
    e5a, _, _ = plan_workload(w5, math_mode=1)
    assert "ewf_acc::exp" in e5a.source()
    w1 = wl.layout_only(wl.c1_affine_tanh)
    e1, _, _ = plan_workload(w1, math_mode=2)
    assert "ewf_fast::tanh" in e1.source()


def test_streaming_hint_only_for_large_operands():
    small, _, _ = plan_workload(wl.layout_only(wl.c4_bias_relu_chansum, n=2))
    assert "ewf_ld_nt" not in small.source()
    big, _, _ = plan_workload(wl.layout_only(wl.c4_bias_relu_chansum))
    assert "ewf_ld_nt<float" in big.source() and "ewf_st_nt<float" in big.source()
    assert "ewf_finish" in big.source()                    # partial sums are folded by a second kernel
    off, _, _ = plan_workload(wl.layout_only(wl.c4_bias_relu_chansum), streaming=2)
    assert "ewf_ld_nt" not in off.source()


def test_structures_beyond_one_kernel_are_planned_in_stages():
    """What no single kernel class covers is split: the reductions that depend on no other are
    materialised by kernels of their own, the rest reads them as broadcastable operands."""
    # reductions over different axis sets in one expression: one stage per set, then nothing is left but copies
    s = GraphSpec(2)
    x = s.input("f32", (False, False))
    s.output(s.reduce("sum", x, (1,)), "f32"); s.output(s.reduce("sum", x, (0,)), "f32")
    expr = ewf.Expression(s)
    ws = expr.plan([ref(BASE, (64, 64))], [ref(BASE + 65536, (64,)), ref(BASE + 131072, (64,))])
    info = expr.info()
    assert info["kernel_class"] == "multi" and info["grid_blocks"] == 3 and ws >= 2 * 64 * 4
    # a value that mixes a cross-row reduction with per-row values needs a grid-wide dependency
    w = wl.layout_only(wl.c3_softmax_xent, rows=8, vocab=16)
    s = w.spec
    loss = s.outputs[3][0]; mean = s.outputs[4][0]
    s.output(s.sub(loss, mean), "f32")
    expr = ewf.Expression(s)
    ins = [ref(BASE, (8, 16)), ref(BASE + 4096, (8, 1))]
    outs = [ref(BASE + 8192 + 512 * k, sh) for k, sh in enumerate(expr.output_shapes(ins))]
    expr.plan(ins, outs)
    assert expr.info()["kernel_class"] == "multi"
    # the gradient of a product over a whole vector: count of zeros and product of the others, then the element-wise part
    s = GraphSpec(1)
    xx = s.input("f32", (False,))
    (gx,) = s.grad([s.reduce("prod", xx, (0,), keep=True)], [s.const(1.0)], [xx])
    s.output(gx, "f32")
    expr = ewf.Expression(s)
    expr.plan([ref(BASE, (1 << 20,))], [ref(BASE + (1 << 30), (1 << 20,))])
    assert expr.info()["kernel_class"] == "multi" and expr.info()["grid_blocks"] == 2


def test_elementwise_outputs_ride_along_the_first_full_pass():
    """Bias + ReLU + per-channel sums on feature maps with short planes: two passes.  The pass that
    materialises the first partial sums walks the whole tensor and writes the element-wise output
    on its way, unless that output lies over an input; which axes go first depends on the plane."""
    def plan(shape, in_place=False, **opts):
        n, c, h, w = shape
        s = GraphSpec(4)
        x = s.input("f32", (False,) * 4); b = s.input("f32", (True, False, True, True))
        y = s.apply("max", s.const(0.0), s.add(x, b))
        s.output(y, "f32"); s.output(s.reduce("sum", y, (0, 2, 3)), "f32")
        e = ewf.Expression(s, **opts)
        xr = ref(BASE, shape)
        e.plan([xr, ref(BASE + (1 << 34), (1, c, 1, 1))], [xr if in_place else ref(BASE + (1 << 35), shape), ref(BASE + (1 << 36), (c,))])
        return e
    for shape, first in (((128, 1024, 14, 14), "lane"), ((128, 512, 28, 28), "lane"), ((64, 288, 36, 36), "row"), ((32, 2048, 7, 7), "col"), ((128, 96, 14, 14), "col")):
        e = plan(shape)
        n, c, h, w = shape
        assert e.info()["kernel_class"] == "multi" and e.info()["grid_blocks"] == 2, (shape, e.info())
        assert e.info(0)["kernel_class"] == first and e.info(0)["extent"] == (n, c, h * w), (shape, e.info(0))
        assert len(e.info(1)["extent"]) == 2, (shape, e.info(1))                   # the second pass sees the small result only
        assert "out0" in e.source(0) and "out1" in e.source(0)
    # in place: the last pass writes the element-wise output, after every pass has read the input
    e = plan((128, 1024, 14, 14), in_place=True)
    assert e.info(1)["extent"] == (128, 1024, 196) and "out1" not in e.source(0)
    # long planes never needed two passes
    assert plan((128, 64, 112, 112)).info()["kernel_class"] == "tile_reduce"


def test_run_argument_checks_without_device():
    expr = _add2()
    ins = [ref(BASE, (3, 4)), ref(BASE + (1 << 20), (1, 4))]
    out = [ref(BASE + (2 << 20), (3, 4))]
    with pytest.raises(ewf.EwfError) as e:
        ewf.run(expr.handle, ins, [1.0], out)                  # the graph has no run-time scalar
    assert e.value.status == ewf.EINVAL
    # a reduce plan needs a workspace of the planned size
    w = wl.layout_only(wl.c4_bias_relu_chansum, n=2)
    e4, ws, _ = plan_workload(w)
    assert ws > 0


def test_distinct_executables_plan_concurrently():
    # the library promises thread safety across distinct executables: the run-time compiler and
    # the code caches are shared, error text is per thread
    import threading
    ops = ["tanh", "exp", "sigmoid", "sqrt", "abs", "neg", "log1p", "sqr"]
    results, errors = {}, []

    def work(i):
        try:
            s = GraphSpec(2)
            x = s.input("f32", (False, False)); b = s.input("f32", (True, False))
            s.output(s.add(s.apply(ops[i % len(ops)], x), b), "f32")
            s.output(s.reduce("sum", x, (1,)), "f32")
            e = ewf.Expression(s)
            ws = e.plan([ref(BASE, (1000 + i % 2, 64)), ref(BASE + (1 << 30), (1, 64))],
                        [ref(BASE + (2 << 30), (1000 + i % 2, 64)), ref(BASE + (3 << 30), (1000 + i % 2,))])
            results[i] = (e.info()["kernel_class"], ws, e.source())
            if i % 4 == 0:                      # and an error on this thread only
                with pytest.raises(ewf.EwfError) as err:
                    e.plan([ref(BASE, (10, 64)), ref(BASE + (1 << 30), (1, 63))], [ref(BASE + (2 << 30), (10, 64)), ref(BASE + (3 << 30), (10,))])
                assert err.value.status == ewf.ESHAPE
        except Exception as ex:                 # noqa: BLE001 - reported below
            errors.append((i, repr(ex)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(16)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    assert len(results) == 16
    # distinct sources were in the compiler at the same time (the lock covers the tables only)
    assert ewf.debug_peak_concurrent_compiles() >= 2
    for i in range(16):
        assert results[i][0] == "row" and (ops[i % len(ops)] in results[i][2] or ops[i % len(ops)] in ("neg", "abs", "sqr", "sqrt"))
        assert results[i][2] == results[(i + 8) % 16][2] or i % 2 != (i + 8) % 2     # same description and layout: same source


def test_prepared_sequence_stops_at_the_failing_call():
    import ctypes
    s = GraphSpec(1)
    x = s.input("f32", (False,)); a = s.scalar("f32")
    s.output(s.mul(x, a), "f32")
    e = ewf.Expression(s)
    tin = ref(BASE, (64,)); tout = ref(BASE + 4096, (64,))
    good = e.bind([tin], [tout], (2.0,), None, 0)
    bad = e.bind([tin], [tout], (), None, 0)               # the scalar is missing: refused before any launch
    seq = ewf.CallSequence([bad])
    with pytest.raises(ewf.EwfError) as err:
        seq.launch()
    assert err.value.status == ewf.EINVAL and err.value.message.startswith("call 0:")
    with pytest.raises(ewf.EwfError) as err:
        bad.launch()
    assert err.value.status == ewf.EINVAL and "scalar" in err.value.message
    assert ewf._lib.ewf_run_sequence(None, 0, None) == 0    # an empty sequence is a no-op
    assert ewf._lib.ewf_run_sequence(None, 3, None) == ewf.EINVAL
    assert ewf._lib.ewf_run_call(None) == ewf.EINVAL
    del good


def test_stages_inherit_the_extent_of_an_axis_only_an_index_spans():
    # max over both axes of the column index, beside a reduction over another set of axes: the
    # stage that reduces the index reads no input, so the extent of its axis comes from the whole expression
    s = GraphSpec(2)
    x = s.input("f32", (False, False))
    s.output(s.reduce("max", s.iota(1), (0, 1), keep=True), "i32")
    s.output(s.reduce("min", x, (0,)), "f32")
    s.output(s.iota(0), "i32")                                      # an output that is an index: shape [rows, 1]
    e = ewf.Expression(s)
    ins = [ref(BASE, (3, 64))]
    assert e.output_shapes(ins) == [(1, 1), (64,), (3, 1)]
    e.plan(ins, [ref(BASE + 4096, (1, 1)), ref(BASE + 8192, (64,)), ref(BASE + 12288, (3, 1))])
    info = e.info()
    assert info["kernel_class"] == "multi"
    stages = [(e.info(k)["extent"], e.source(k)) for k in range(info["grid_blocks"])]
    index_stage = [ext for ext, src in stages if "p.in0" not in src.split("ewf_kernel", 1)[1]]
    assert index_stage and all(int(np.prod(ext)) == 64 for ext in index_stage), [ext for ext, _ in stages]   # 64 columns, not a single element


def test_an_input_no_output_uses_is_never_read():
    # a permuted operand would be staged through LDS, but nothing uses it: it must not appear in the kernel
    s = GraphSpec(2)
    unused = s.input("f32", (False, False)); y = s.input("i32", (False, False))
    s.apply("tanh", unused)
    s.output(y, "i32")
    e = ewf.Expression(s, block_threads=64)
    e.plan([ref(BASE, (512, 300), (1, 512)), ref(BASE + (1 << 30), (512, 300))], [ref(BASE + (2 << 30), (512, 300))])
    assert e.info()["staged_operands"] == 0 and "q_in0" not in e.source()


# ------------------------------------------------------------------ the ABI's exception barrier

def test_no_exception_crosses_the_abi():
    """Faults injected where the library asks for host memory come back as status codes with a
    message, from graph building, compilation, planning and the gradient call alike; the handles
    stay usable afterwards."""
    g = ewf.graph_create(2)
    x = ewf.input(g, ewf.F32, [0, 0])
    for kind, status, text in ((1, ewf.ENOMEM, "memory"), (2, ewf.EINVAL, "injected fault")):
        ewf.debug_inject_fault(kind, 0)
        with pytest.raises(ewf.EwfError) as err:
            ewf.apply(g, ewf.OPS["tanh"], [x])
        assert err.value.status == status and text in err.value.message
    y = ewf.apply(g, ewf.OPS["tanh"], [x])                 # the fault fired once; the graph is intact
    assert y == x + 1
    # inside ewf_grad, a few nodes into the traversal
    ewf.debug_inject_fault(1, 2)
    with pytest.raises(ewf.EwfError) as err:
        ewf.grad(g, [y], [ewf.const(g, ewf.F32, 1.0)], [x])
    assert err.value.status == ewf.ENOMEM
    ewf.debug_inject_fault(0, 0)
    ewf.output(g, y, ewf.F32)
    e = ewf.compile(g)
    ewf.graph_destroy(g)
    ins = [ref(BASE, (8, 16))]; outs = [ref(BASE + (1 << 30), (8, 16))]
    for kind, status in ((1, ewf.ENOMEM), (2, ewf.EINVAL)):
        ewf.debug_inject_fault(kind, 0)
        with pytest.raises(ewf.EwfError) as err:
            ewf.plan(e, ins, outs)
        assert err.value.status == status
    assert ewf.plan(e, ins, outs) == 0 and ewf.debug_plan_info(e)["kernel_class"] == "tile"
    # the run call passes the same point before it touches the device
    ewf.debug_inject_fault(2, 0)
    with pytest.raises(ewf.EwfError) as err:
        ewf.run(e, ins, [], outs)
    assert err.value.status == ewf.EINVAL and "injected" in err.value.message
    ewf.debug_inject_fault(0, 0)
    ewf.exec_destroy(e)


def test_an_empty_plan_checks_the_pointers_it_fills_on_every_call():
    # a sum over an empty axis is filled with 0 by a kernel: a plan found in the cache must
    # refuse a null output pointer just as the first call does
    s = GraphSpec(2)
    s.output(s.reduce("sum", s.input("f32", (False, False)), (1,)), "f32")
    e = ewf.Expression(s)
    ins = [ref(BASE, (5, 0))]
    assert e.plan(ins, [ref(BASE + (1 << 30), (5,))]) == 0
    with pytest.raises(ewf.EwfError) as err:
        e.plan(ins, [ref(0, (5,))])
    assert err.value.status == ewf.EINVAL and "null" in err.value.message
    with pytest.raises(ewf.EwfError) as err:
        e.run(ins, [ref(0, (5,))])
    assert err.value.status == ewf.EINVAL
