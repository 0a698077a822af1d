// C ABI: compile / plan / run, the per-layout plan cache and the introspection calls.
//
// ewf_run follows the rule the paper draws from its allocator experience (section 3.1.3:
// freeing device memory synchronises the device): the hot call allocates nothing on the
// device, frees nothing and never synchronises; it only patches pointers and scalars into a
// prepared argument block and enqueues one kernel on the caller's stream (section 3.1.5:
// computations are asynchronous so the host can run ahead).
#include <hip/hip_runtime.h>

// (declared here: the runtime's extension header needs the device compiler's front end)
extern "C" hipError_t hipExtModuleLaunchKernel(hipFunction_t f, uint32_t globalWorkSizeX, uint32_t globalWorkSizeY,
                                               uint32_t globalWorkSizeZ, uint32_t localWorkSizeX, uint32_t localWorkSizeY,
                                               uint32_t localWorkSizeZ, size_t sharedMemBytes, hipStream_t hStream,
                                               void **kernelParams, void **extra, hipEvent_t startEvent, hipEvent_t stopEvent,
                                               uint32_t flags);

#include <cstring>

#include "ewf_internal.h"

namespace ewf {
const Graph &graph_of(const ewf_graph *g);
void aux_fill_zero(void *ptr, size_t nbytes, hipStream_t stream);
void aux_copy(void *dst, const void *src, size_t nbytes, hipStream_t stream);
void aux_fill_view(void *ptr, int rank, const int64_t *shape, const int64_t *strides, int elem_bytes, uint32_t bits,
                   hipStream_t stream);
}  // namespace ewf

using namespace ewf;

namespace {

std::string layout_signature(const Graph &g, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout)
{
    std::string s;
    auto put = [&](int64_t v) { s.append(reinterpret_cast<const char *>(&v), 8); };
    for (int k = 0; k < nin; k++) {
        for (int d = 0; d < g.ndim; d++) { put(in[k].shape[d]); put(in[k].strides[d]); }
        put((int64_t)((uintptr_t)in[k].ptr & 15));
    }
    for (int k = 0; k < nout; k++) {
        const Node &v = g.nodes[g.outputs[k].value];
        int orank = g.ndim - __builtin_popcount(v.dropped);
        for (int d = 0; d < orank; d++) { put(out[k].shape[d]); put(out[k].strides[d]); }
        put((int64_t)((uintptr_t)out[k].ptr & 15));
        // exact aliasing of an input changes nothing in the kernel but must be re-validated
        int alias = -1;
        for (int j = 0; j < nin; j++) if (in[j].ptr == out[k].ptr) alias = j;
        put(alias);
    }
    return s;
}

bool args_present(const Graph &g, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout)
{
    if (nin != g.ninputs || nout != (int)g.outputs.size()) return false;
    if ((nin > 0 && !in) || (nout > 0 && !out)) return false;
    for (int k = 0; k < nin; k++) if (g.ndim > 0 && (!in[k].shape || !in[k].strides)) return false;
    for (int k = 0; k < nout; k++) {
        const Node &v = g.nodes[g.outputs[k].value];
        int orank = g.ndim - __builtin_popcount(v.dropped);
        if (orank > 0 && (!out[k].shape || !out[k].strides)) return false;
    }
    return true;
}

}  // namespace

namespace ewf {

// Measurement aid: pairs of events, each tied to one dispatch of a main kernel (they carry that
// dispatch's own begin and end time stamps, unlike events recorded around a launch call).
struct KernelTiming {
    std::vector<hipEvent_t> start, stop;
    int used = 0;
    ~KernelTiming()
    {
        for (hipEvent_t ev : start) (void)hipEventDestroy(ev);
        for (hipEvent_t ev : stop) (void)hipEventDestroy(ev);
    }
};

static ewf_status single_kernel_plan(Exec &e, Plan *plan, const int64_t *full);
constexpr int kMaxKernelArgBytes = 4096;           // what the hardware's kernel-argument segment holds

ewf_status make_plan(Exec &e, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout, Plan **result, bool lookup_only)
{
    if (!args_present(e.g, in, nin, out, nout)) {
        set_error("expected %d input and %d output tensors with shape and strides", e.g.ninputs, (int)e.g.outputs.size());
        return EWF_EINVAL;
    }
    fault_point();
    std::string sig = layout_signature(e.g, in, nin, out, nout);
    auto it = e.plans.find(sig);
    if (it != e.plans.end()) {
        // same shapes, strides and alignment; only the pointers may differ from the planning
        // call, and the aliasing rules depend on them
        Plan *p = it->second.get();
        bool same = true;
        for (int k = 0; k < nin; k++) same = same && p->raw[k].addr == (uint64_t)(uintptr_t)in[k].ptr;
        for (int k = 0; k < nout; k++) same = same && p->raw[nin + k].addr == (uint64_t)(uintptr_t)out[k].ptr;
        if (!same) {
            for (int k = 0; k < nin; k++) p->raw[k].addr = (uint64_t)(uintptr_t)in[k].ptr;
            for (int k = 0; k < nout; k++) p->raw[nin + k].addr = (uint64_t)(uintptr_t)out[k].ptr;
            if (!p->empty)
                for (int k = 0; k < nin + nout; k++)
                    if (!p->raw[k].addr) { p->raw[0].addr = ~(uint64_t)0; set_error("operand %d: null pointer", k); return EWF_EINVAL; }
            // nothing to traverse, but outputs that are sums or products over the empty axis are
            // still filled: those need memory behind them
            for (const Plan::Fill &f : p->fills)
                if (!p->raw[nin + f.output].addr) { p->raw[0].addr = ~(uint64_t)0; set_error("output %d: null pointer", f.output); return EWF_EINVAL; }
            for (const Stage &sg : p->stages)
                for (int d : sg.out_dst)
                    if (d >= 0 && !p->raw[nin + d].addr) { p->raw[0].addr = ~(uint64_t)0; set_error("output %d: null pointer", d); return EWF_EINVAL; }
            ewf_status st = check_aliasing(p->raw, nin, nout);
            if (st != EWF_OK) { p->raw[0].addr = ~(uint64_t)0; return st; }
        }
        e.last = p;
        *result = p;
        return EWF_OK;
    }

    if (lookup_only) {
        set_error("this layout has not been planned: call ewf_plan for it first (this entry point compiles nothing)");
        return EWF_EINVAL;
    }
    std::unique_ptr<Plan> plan(new Plan());
    int64_t full[kMaxDims];
    ewf_status st = infer_full_extents(e.g, in, nin, full, e.has_forced_full ? e.forced_full : nullptr);
    if (st != EWF_OK) return st;
    uint32_t unit = 0;
    bool empty = false;
    for (int d = 0; d < e.g.ndim; d++) { if (full[d] == 1) unit |= 1u << d; if (full[d] == 0) empty = true; }
    // an arg-max is an int32 position among the elements it ranks
    for (const Node &nd : e.g.nodes) {
        if (nd.kind != NodeKind::Reduce || nd.op != EWF_RARGMAX) continue;
        int64_t positions = 1;
        for (int d = 0; d < e.g.ndim; d++)
            if ((nd.axes >> d & 1u) && !(e.g.nodes[nd.args[0]].bcast >> d & 1u)) positions *= std::max<int64_t>(full[d], 1);
        if (positions > 2147483647) { set_error("arg-max over %lld positions does not fit its int32 result", (long long)positions); return EWF_ESHAPE; }
    }
    plan->red = analyse_reductions(e.g, unit);
    st = canonicalize(e, plan->red, in, nin, out, nout, true, plan->canon, full, &plan->raw);
    if (st != EWF_OK) return st;

    if (empty) {
        // nothing to traverse; reductions over an empty axis still define their outputs
        std::vector<int> rest;                          // outputs computed from such reductions
        for (size_t k = 0; k < e.g.outputs.size(); k++) {
            const Node &v = e.g.nodes[e.g.outputs[k].value];
            bool out_empty = false;
            for (int d = 0; d < e.g.ndim; d++)
                if (!(v.bcast & (1u << d)) && full[d] == 0) out_empty = true;
            if (!out_empty) {
                // a reduction over an empty axis: sum and product have an identity, the others do not
                const int orank = e.g.ndim - __builtin_popcount(v.dropped);
                uint32_t bits = 0;
                bool ok = v.kind == NodeKind::Reduce && (v.op == EWF_RSUM || v.op == EWF_RPROD);
                if (ok && v.op == EWF_RPROD) {
                    if (e.g.outputs[k].storage == EWF_I32) bits = 1;
                    else if (e.g.outputs[k].storage == EWF_F16) bits = 0x3c00u;
                    else bits = 0x3f800000u;
                }
                if (!ok) { rest.push_back((int)k); continue; }
                plan->fills.push_back({(int)k, orank, e.g.outputs[k].storage == EWF_F16 ? 2 : 4, bits});
            }
        }
        if (!rest.empty()) {
            st = plan_empty_rest(e, full, in, nin, out, nout, rest, *plan);
            if (st != EWF_OK) return st;
        }
        plan->empty = true;
        plan->kclass = rest.empty() ? KernelClass::None : KernelClass::Multi;
        plan->grid = (int64_t)plan->stages.size();
        e.last = plan.get();
        *result = e.last;
        e.plans.emplace(sig, std::move(plan));
        return EWF_OK;
    }

    plan->avoid_poor_rows = !e.is_stage || e.strict_rows;
    {
        Graph fused = e.g;
        plan->fused_depth = fuse_shifted_exp_sums(fused) > 0 ? analyse_reductions(fused, unit).max_depth : plan->red.max_depth;
    }
    plan->avoid_short_runs = !e.is_stage;
    st = single_kernel_plan(e, plan.get(), full);
    if (st == EWF_EUNSUPPORTED && !e.is_stage) {
        // no single kernel covers the expression (or only a poorly fitting one does): several
        // passes, reductions materialised; a softmax-style chain max -> sum of exp first
        // becomes one level, reductions over axes far apart in memory are taken in two steps
        const std::string why = get_error();
        const bool refused = plan->row_refused || plan->axes_refused;
        Graph split = e.g;
        fuse_shifted_exp_sums(split);
        // likewise mean -> sum of squared deviations from it: one sweep instead of two
        if (!e.opts.no_rewrite) fuse_centred_squares(split, full);
        if (plan->axes_refused && split_reduction_axes(split, plan->red.axes, plan->split_first_axes) < 0) split = e.g;
        st = plan_multi(e, split, true, in, nin, out, nout, *plan);
        if (st == EWF_EUNSUPPORTED) {
            plan->stages.clear();
            plan->temps.clear();
            if (refused) {
                // the single kernel after all
                plan->avoid_poor_rows = false;
                plan->avoid_short_runs = false;
                plan->row_refused = plan->axes_refused = false;
                st = single_kernel_plan(e, plan.get(), full);
            } else {
                st = plan_multi(e, split, false, in, nin, out, nout, *plan);
                if (st == EWF_EUNSUPPORTED) set_error_str(why + "; and a plan in several passes failed: " + get_error());
                if (st == EWF_OK) plan->kclass = KernelClass::Multi;
            }
        } else if (st == EWF_OK) {
            plan->kclass = KernelClass::Multi;
        }
    }
    if (st != EWF_OK) return st;
    e.last = plan.get();
    *result = e.last;
    e.plans.emplace(sig, std::move(plan));
    return EWF_OK;
}

static ewf_status single_kernel_plan(Exec &e, Plan *plan, const int64_t *full)
{
    ewf_status st = EWF_OK;
    const Canon &c = plan->canon;
    bool row_only = false;                     // only the row class covers the expression
    bool cross_only = false;                   // ... and only because of reductions over the rows
    if (!plan->red.has_reduce) {
        plan->kclass = KernelClass::Tile;
    } else {
        if (!plan->red.unsupported.empty()) { set_error("unsupported reduction structure: %s", plan->red.unsupported.c_str()); return EWF_EUNSUPPORTED; }
        int nred = 0;
        for (int d = 0; d < c.rank; d++) nred += c.reduced[d];
        const bool inner_only = nred == 1 && c.reduced[c.rank - 1];
        int64_t rows = 1;
        for (int d = 0; d < c.rank - 1; d++) rows *= c.extent[d];
        const bool needs_row = plan->red.max_depth > 1 || !plan->red.cross_nodes.empty();
        bool full_dep_out = false;             // an output that varies along the row and uses a reduction
        for (const OutputDecl &od : e.g.outputs)
            if (plan->red.edepth[od.value] >= 1 && (e.g.nodes[od.value].bcast & plan->red.axes) != plan->red.axes) full_dep_out = true;
        if (!c.reduced[c.rank - 1]) {
            // the reduced axes are not the fastest-varying ones in memory: column class
            if (needs_row || full_dep_out) {
                set_error("unsupported: chained or cross-group reductions need the reduced axes to form the innermost contiguous dimension");
                return EWF_EUNSUPPORTED;
            }
            plan->kclass = KernelClass::Col;
        } else if (needs_row || full_dep_out) {
            if (!inner_only) {
                set_error("unsupported: chained or cross-group reductions need the reduced axes to form the innermost contiguous dimension");
                return EWF_EUNSUPPORTED;
            }
            if (!plan->red.cross_nodes.empty() && rows > 65536 && (!e.is_stage || e.strict_rows)) {
                // one workgroup folds the per-row values of a cross-row reduction: beyond some
                // ten thousand rows a separate, parallel reduction over them is faster
                set_error("unsupported: too many rows for the single-workgroup fold of a cross-row reduction");
                return EWF_EUNSUPPORTED;
            }
            if (!plan->red.cross_nodes.empty()) {
                // the cross-group reduction must fold every remaining group
                for (int d = 0; d < e.g.ndim; d++) {
                    bool varies = full[d] > 1 && !(plan->red.axes & (1u << d));
                    if (varies && !(plan->red.cross_axes & (1u << d))) {
                        set_error("unsupported: the second reduction must cover every axis the first one keeps");
                        return EWF_EUNSUPPORTED;
                    }
                }
            }
            plan->kclass = KernelClass::Row;
            row_only = true;
            cross_only = plan->red.max_depth <= 1 && !full_dep_out && rows <= 8192;
        } else if (inner_only && rows >= 512 && c.extent[c.rank - 1] <= 65536) {
            plan->kclass = KernelClass::Row;
        } else {
            plan->kclass = KernelClass::TileReduce;
            // Reduced axes that are not neighbours in memory: kk is the innermost kept dimension
            // with reduced dimensions on both sides.  When the run inside it is short, the tiles
            // (which never leave a reduction group) would be tiny.
            int kk = -1;
            bool seen_reduced = false;
            for (int d = 0; d < c.rank; d++) {
                if (c.reduced[d]) seen_reduced = true;
                else if (seen_reduced) kk = d;
            }
            if (plan->avoid_short_runs && kk >= 0 && kk < c.rank - 1 && c.total >= ((int64_t)1 << 20)) {
                int64_t inner = 1, outer = 1;
                for (int d = 0; d < c.rank; d++) if (c.reduced[d]) (d > kk ? inner : outer) *= c.extent[d];
                bool ops_ok = true;
                for (int n : plan->red.level_nodes) {
                    const Node &nd = e.g.nodes[n];
                    ops_ok = ops_ok && nd.axes == plan->red.axes &&
                             (nd.op == EWF_RSUM || nd.op == EWF_RPROD || nd.op == EWF_RMAX || nd.op == EWF_RMIN);
                }
                uint32_t outer_axes = 0, inner_axes = 0;
                for (int a = 0; a < e.g.ndim; a++) {
                    if (!(plan->red.axes >> a & 1u) || c.dim_of_axis[a] < 0) continue;
                    (c.dim_of_axis[a] < kk ? outer_axes : inner_axes) |= 1u << a;
                }
                if (ops_ok && inner < 2048 && outer >= 2 && outer_axes) {
                    plan->axes_refused = true;
                    // Which axes the first pass takes.  The outer ones leave a column kernel whose
                    // columns are the kept and the inner dimensions; the inner ones leave short
                    // contiguous rows, several to a wavefront, which is the faster sweep once a
                    // run is a cache line and a half and the tensor is large (bias + ReLU +
                    // per-channel sums, float32 [128, 1024, 14, 14]: 37 against 52 us; [128, 2048,
                    // 7, 7]: 35 against 45 us; but float16 [128, 2048, 7, 7]: 36 against 23 us, and
                    // float32 [32, 2048, 7, 7]: 13 against 9.5 us).
                    int in_sz = 4;
                    for (size_t k = 0; k < c.ops.size(); k++)
                        if (!c.ops[k].is_output && c.ops[k].stride[c.rank - 1] != 0) in_sz = std::min(in_sz, c.ops[k].storage == EWF_F16 ? 2 : 4);
                    const bool inner_first = inner * in_sz >= 192 && c.total >= ((int64_t)1 << 23) && inner_axes;
                    plan->split_first_axes = inner_first ? inner_axes : outer_axes;
                    set_error("the reduced axes are not neighbours in memory and the innermost run is short (%lld elements)", (long long)inner);
                    return EWF_EUNSUPPORTED;
                }
            }
        }
    }

    if (plan->kclass == KernelClass::Row) {
        // rows of up to 4096 bytes, many of them: several rows per wavefront, or a wavefront per row
        // and four rows per workgroup, instead of a workgroup per row (softmax over float32 rows
        // of 1024: 52.8 -> 42.0 us; layer normalisation of [65536, 1000]: 109 -> 78 us).  Sum over float32 rows, 134 MB, row class / lane class in TB/s:
        // 8 columns 0.4 / 6.0, 16: 0.8 / 6.4, 32: 1.5 / 6.7, 64: 2.8 / 6.7, 128: 4.7 / 6.7, 256: 6.1 / 6.6
        int widest = 2;
        for (const Operand &op : c.ops) if (op.stride[c.rank - 1] != 0) widest = std::max(widest, op.storage == EWF_F16 ? 2 : 4);
        int64_t rows_ = 1;
        for (int d = 0; d < c.rank - 1; d++) rows_ *= c.extent[d];
        // (rows that allow only narrow accesses -- an odd length, a misaligned slice -- up to 1024
        // of them per row: the row class, one such access per thread in flight, reads rows of 289
        // float32 at 2.8 TB/s)
        int narrowest = 4;
        for (const Operand &op : c.ops) if (op.stride[c.rank - 1] != 0) narrowest = std::min(narrowest, op.storage == EWF_F16 ? 2 : 4);
        const bool narrow = c.vec * narrowest < 16;
        const bool short_rows = c.extent[c.rank - 1] * widest <= 4096 || (narrow && c.extent[c.rank - 1] / c.vec <= 1024);
        if (short_rows && rows_ >= 4096 && e.opts.split_rows != 1) {
            plan->kclass = KernelClass::Lane;
            st = generate(e, *plan);
            if (st == EWF_EUNSUPPORTED) plan->kclass = KernelClass::Row;      // e.g. too many row operands for one thread
        }
    }
    if (plan->kclass != KernelClass::Lane) st = generate(e, *plan);
    if (st == EWF_EUNSUPPORTED && plan->row_refused && plan->kclass == KernelClass::Row && (!row_only || cross_only)) {
        // plain row reductions do not need the row class, nor does a single level of them followed
        // by reductions over the rows (those are folded by the finish kernel)
        const std::string why = get_error();
        plan->kclass = KernelClass::TileReduce;
        st = generate(e, *plan);
        if (st == EWF_OK) plan->row_refused = false;
        else if (row_only) { plan->kclass = KernelClass::Row; set_error_str(why); }
    }
    if (st != EWF_OK) return st;
    if (plan->args.size() > kMaxKernelArgBytes) {
        set_error("unsupported: the kernel's argument block would take %zu bytes (at most %d): too many operands or dimensions for one kernel",
                  plan->args.size(), kMaxKernelArgBytes);
        return EWF_EUNSUPPORTED;
    }
    bool cached = false;
    st = compile_source(plan->source, plan->code, &cached);
    if (st != EWF_OK) return st;
    if (!cached) e.compile_count++;
    if (plan->used_auto_occupancy && code_scratch_bytes(plan->code) > 0) {
        // the register budget the generator asked for made the compiler spill: a second round
        // of workgroups costs less than scratch traffic, so generate again without it
        plan->no_auto_occupancy = true;
        plan->used_auto_occupancy = false;
        plan->layout = ParamLayout();
        st = generate(e, *plan);
        if (st != EWF_OK) return st;
        st = compile_source(plan->source, plan->code, &cached);
        if (st != EWF_OK) return st;
        if (!cached) e.compile_count++;
    }
    return EWF_OK;
}

}  // namespace ewf

extern "C" {

ewf_status ewf_compile(const ewf_graph *g, const ewf_options *opts, ewf_exec **out)
{
    return guarded([&]() -> ewf_status {
        if (!g || !out) { set_error("null argument"); return EWF_EINVAL; }
        ewf_exec *x = new (std::nothrow) ewf_exec();
        if (!x) return EWF_ENOMEM;
        x->e.g = graph_of(g);
        if (opts) x->e.opts = *opts;
        ewf_status st = finalize_graph(x->e.g);
        if (st != EWF_OK) { delete x; return st; }
        x->e.nodes_before = (int)x->e.g.nodes.size();
        if (!x->e.opts.no_rewrite) {
            rewrite_graph(x->e.g);
            // (The chain max -> sum of exp(x - max) stays two levels here.  As one rescaled level it
            // saves a sweep only where rows are split over workgroups, and the planner makes it one
            // there; over rows held in registers the rescaled update costs more per element than it
            // saves: softmax probabilities, float16 [131072, 512] 65 us fused against 41 us, float32
            // [1048576, 64] 100 against 79 us, the gradient of softmax cross-entropy on [1280, 10000]
            // 21.0 against 21.2 us.)
            st = finalize_graph(x->e.g);
            if (st != EWF_OK) { delete x; return st; }
        }
        x->e.nodes_after = (int)x->e.g.nodes.size();
        bool all_f16 = true;
        for (const OutputDecl &o : x->e.g.outputs) if (o.storage != EWF_F16) all_f16 = false;
        const int mm = x->e.opts.math_mode;
        if (mm < 0 || mm > 3) { delete x; set_error("math_mode must be 0..3"); return EWF_EINVAL; }
        x->e.math_flavour = mm == 0 ? (all_f16 ? 3 : 1) : mm;
        x->e.auto_math = mm == 0;
        *out = x;
        return EWF_OK;
    });
}

void ewf_exec_destroy(ewf_exec *e)
{
    if (e) { delete e->e.timing; e->e.timing = nullptr; }
    delete e;
}

ewf_status ewf_debug_time_kernels(ewf_exec *e, int32_t slots)
{
    return guarded([&]() -> ewf_status {
        if (!e || slots < 0 || slots > (1 << 20)) { set_error("bad argument"); return EWF_EINVAL; }
        delete e->e.timing;
        e->e.timing = nullptr;
        if (slots == 0) return EWF_OK;
        KernelTiming *t = new (std::nothrow) KernelTiming();
        if (!t) return EWF_ENOMEM;
        for (int i = 0; i < slots; i++) {
            hipEvent_t a = nullptr, b = nullptr;
            if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
                if (a) (void)hipEventDestroy(a);
                delete t;
                set_error("hipEventCreate failed");
                return EWF_EHIP;
            }
            t->start.push_back(a); t->stop.push_back(b);
        }
        e->e.timing = t;
        return EWF_OK;
    });
}

ewf_status ewf_debug_kernel_times(ewf_exec *e, float *ms, int32_t capacity, int32_t *count)
{
    return guarded([&]() -> ewf_status {
        if (!e || !count || (capacity > 0 && !ms)) { set_error("null argument"); return EWF_EINVAL; }
        *count = 0;
        KernelTiming *t = e->e.timing;
        if (!t) return EWF_OK;
        for (int i = 0; i < t->used && i < capacity; i++) {
            hipError_t he = hipEventSynchronize(t->stop[i]);
            if (he == hipSuccess) he = hipEventElapsedTime(&ms[i], t->start[i], t->stop[i]);
            if (he != hipSuccess) { set_error("kernel timing: %s", hipGetErrorString(he)); return EWF_EHIP; }
            *count = i + 1;
        }
        t->used = 0;
        return EWF_OK;
    });
}

ewf_status ewf_output_shape(ewf_exec *e, const ewf_tensor *in, int32_t nin, int32_t k, int32_t *rank_out,
                            int64_t *shape_out)
{
    return guarded([&]() -> ewf_status {
        if (!e || !rank_out || !shape_out) { set_error("null argument"); return EWF_EINVAL; }
        const Graph &g = e->e.g;
        if (k < 0 || k >= (int)g.outputs.size()) { set_error("no such output"); return EWF_EINVAL; }
        int64_t full[kMaxDims];
        ewf_status st = infer_full_extents(g, in, nin, full);
        if (st != EWF_OK) return st;
        const Node &v = g.nodes[g.outputs[k].value];
        int r = 0;
        for (int d = 0; d < g.ndim; d++) {
            if (v.dropped & (1u << d)) continue;
            shape_out[r++] = (v.bcast & (1u << d)) ? 1 : full[d];
        }
        *rank_out = r;
        return EWF_OK;
    });
}

ewf_status ewf_plan(ewf_exec *e, const ewf_tensor *in, int32_t nin, const ewf_tensor *out, int32_t nout,
                    size_t *workspace_bytes)
{
    return guarded([&]() -> ewf_status {
        if (!e) { set_error("null executable"); return EWF_EINVAL; }
        Plan *p = nullptr;
        ewf_status st = make_plan(e->e, in, nin, out, nout, &p);
        if (st != EWF_OK) return st;
        if (workspace_bytes) *workspace_bytes = p->workspace_bytes;
        // with a device at hand the kernels are loaded now rather than by the first launch (planning
        // itself needs no device: the run-time compiler cross-compiles)
        int ndev = 0;
        if (hipGetDeviceCount(&ndev) == hipSuccess && ndev > 0) return load_plan_functions(*p);
        (void)hipGetLastError();
        return EWF_OK;
    });
}

ewf_status ewf_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return guarded([&]() -> ewf_status {
        if (workspace_bytes == 0) return EWF_OK;
        if (!workspace || ((uintptr_t)workspace & 15)) { set_error("workspace must be a 16-byte aligned device pointer"); return EWF_EINVAL; }
        aux_fill_zero(workspace, workspace_bytes, (hipStream_t)hip_stream);
        hipError_t he = hipGetLastError();
        if (he != hipSuccess) { set_error("workspace fill: %s", hipGetErrorString(he)); return EWF_EHIP; }
        return EWF_OK;
    });
}

ewf_status ewf_run(ewf_exec *e, const ewf_tensor *in, int32_t nin, const double *scalars, int32_t nscalars,
                   const ewf_tensor *out, int32_t nout, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return guarded([&]() -> ewf_status {
        if (!e) { set_error("null executable"); return EWF_EINVAL; }
        return run_exec(e->e, in, nin, scalars, nscalars, out, nout, workspace, workspace_bytes, hip_stream);
    });
}

}  // extern "C"

namespace ewf {

ewf_status load_plan_functions(Plan &p)
{
    if (p.empty && p.stages.empty()) return EWF_OK;
    if (p.kclass == KernelClass::Multi) {
        for (Stage &sg : p.stages) {
            if (!sg.exec->last) continue;
            ewf_status st = load_plan_functions(*sg.exec->last);
            if (st != EWF_OK) return st;
        }
        return EWF_OK;
    }
    int dev = -1;
    if (p.function && hipGetDevice(&dev) == hipSuccess && dev == p.function_device) return EWF_OK;
    ewf_status st = load_function(p.code, "ewf_kernel", &p.function, &p.function_device);
    if (st != EWF_OK) return st;
    if (p.finish_grid > 0) {
        st = load_function(p.code, "ewf_finish", &p.finish_function, &p.function_device);
        if (st != EWF_OK) { p.function = nullptr; return st; }
    }
    return EWF_OK;
}

ewf_status run_exec(Exec &x, const ewf_tensor *in, int32_t nin, const double *scalars, int32_t nscalars,
                    const ewf_tensor *out, int32_t nout, void *workspace, size_t workspace_bytes, void *hip_stream,
                    bool no_setup)
{
    if (nscalars != x.g.nscalars || (nscalars > 0 && !scalars)) {
        set_error("expected %d run-time scalar(s), got %d", x.g.nscalars, nscalars);
        return EWF_EINVAL;
    }
    Plan *p = nullptr;
    ewf_status st = make_plan(x, in, nin, out, nout, &p, no_setup);
    if (st != EWF_OK) return st;
    if (p->empty) {
        for (const Plan::Fill &f : p->fills) {
            aux_fill_view(out[f.output].ptr, f.rank, out[f.output].shape, out[f.output].strides, f.elem_bytes, f.bits,
                          (hipStream_t)hip_stream);
            hipError_t he = hipGetLastError();
            if (he != hipSuccess) { set_error("fill launch: %s", hipGetErrorString(he)); return EWF_EHIP; }
        }
        if (p->stages.empty()) return EWF_OK;
        // values computed from reductions over an empty axis: the reductions are temporaries set
        // to their identity, then one stage computes the outputs
        if (!workspace || workspace_bytes < p->workspace_bytes) {
            set_error("workspace of %zu bytes needed, %zu given", p->workspace_bytes, workspace ? workspace_bytes : (size_t)0);
            return EWF_ENOMEM;
        }
        if ((uintptr_t)workspace & 15) { set_error("workspace must be 16-byte aligned"); return EWF_EINVAL; }
        for (const Plan::TempFill &tf : p->temp_fills) {
            const Temp &t = p->temps[tf.temp];
            aux_fill_view((char *)workspace + t.offset, x.g.ndim, t.shape, t.strides, 4, tf.bits, (hipStream_t)hip_stream);
            hipError_t he = hipGetLastError();
            if (he != hipSuccess) { set_error("fill launch: %s", hipGetErrorString(he)); return EWF_EHIP; }
        }
        return run_multi(x, *p, in, nin, scalars, nscalars, out, nout, workspace, workspace_bytes, hip_stream, no_setup);
    }
    if (p->workspace_bytes > 0) {
        if (!workspace || workspace_bytes < p->workspace_bytes) {
            set_error("workspace of %zu bytes needed, %zu given", p->workspace_bytes, workspace ? workspace_bytes : (size_t)0);
            return EWF_ENOMEM;
        }
        if ((uintptr_t)workspace & 15) { set_error("workspace must be 16-byte aligned"); return EWF_EINVAL; }
    }
    if (p->kclass == KernelClass::Multi)
        return run_multi(x, *p, in, nin, scalars, nscalars, out, nout, workspace, workspace_bytes, hip_stream, no_setup);
    int dev = -1;
    if (!p->function || hipGetDevice(&dev) != hipSuccess || dev != p->function_device) {
        if (no_setup) {
            set_error("the kernels of this layout are not loaded on the current device: call ewf_plan with that device current first");
            return EWF_EINVAL;
        }
        st = load_plan_functions(*p);
        if (st != EWF_OK) return st;
    }

    // patch pointers and scalars into a copy of the prepared argument block
    // (a kernel takes at most 4 KiB of arguments: layouts beyond that are refused when planned,
    // so the copy always fits the stack and a launch allocates nothing)
    uint8_t args[kMaxKernelArgBytes];
    if (p->args.size() > sizeof args) { set_error("argument block of %zu bytes", p->args.size()); return EWF_EUNSUPPORTED; }
    memcpy(args, p->args.data(), p->args.size());
    const ParamLayout &L = p->layout;
    size_t f = 0;
    for (int k = 0; k < nin; k++, f++) memcpy(args + L.offsets[f], &in[k].ptr, 8);
    for (int k = 0; k < nout; k++, f++) memcpy(args + L.offsets[f], &out[k].ptr, 8);
    void *partials = workspace;
    memcpy(args + L.offsets[f++], &partials, 8);
    for (int k = 0; k < nscalars; k++) {
        size_t fi = L.fields.size() - (size_t)nscalars + (size_t)k;
        if (L.fields[fi].type == ParamField::I32) { int32_t v = (int32_t)scalars[k]; memcpy(args + L.offsets[fi], &v, 4); }
        else { float v = (float)scalars[k]; memcpy(args + L.offsets[fi], &v, 4); }
    }
    size_t arg_size = p->args.size();
    void *config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, args, HIP_LAUNCH_PARAM_BUFFER_SIZE, &arg_size, HIP_LAUNCH_PARAM_END};
    hipError_t he;
    KernelTiming *tm = x.timing;
    if (tm && tm->used < (int)tm->start.size() && p->grid * p->block < ((int64_t)1 << 32)) {
        // a timed run: the same launch with a pair of events attached to this dispatch
        const int slot = tm->used++;
        he = hipExtModuleLaunchKernel((hipFunction_t)p->function, (uint32_t)(p->grid * p->block), 1, 1, (uint32_t)p->block, 1, 1, 0,
                                      (hipStream_t)hip_stream, nullptr, config, tm->start[slot], tm->stop[slot], 0);
    } else {
        he = hipModuleLaunchKernel((hipFunction_t)p->function, (unsigned)p->grid, 1, 1, (unsigned)p->block, 1, 1,
                                   0 /* LDS is declared statically in the kernels */, (hipStream_t)hip_stream, nullptr, config);
    }
    if (he != hipSuccess) { set_error("kernel launch: %s", hipGetErrorString(he)); return EWF_EHIP; }
    if (p->finish_grid > 0) {
        // partial results are folded by a second kernel on the same stream
        he = hipModuleLaunchKernel((hipFunction_t)p->finish_function, (unsigned)p->finish_grid, 1, 1,
                                   (unsigned)p->finish_block, 1, 1, 0, (hipStream_t)hip_stream, nullptr, config);
        if (he != hipSuccess) { set_error("kernel launch (fold): %s", hipGetErrorString(he)); return EWF_EHIP; }
    }
    return EWF_OK;
}

}  // namespace ewf

extern "C" {

ewf_status ewf_run_call(const ewf_call *c)
{
    return guarded([&]() -> ewf_status {
        if (!c) { set_error("null argument"); return EWF_EINVAL; }
        return ewf_run(c->exec, c->in, c->nin, c->scalars, c->nscalars, c->out, c->nout, c->workspace, c->workspace_bytes,
                       c->hip_stream);
    });
}

ewf_status ewf_run_sequence(const ewf_call *calls, int32_t ncalls, int32_t *failed)
{
    return guarded([&]() -> ewf_status {
        if (ncalls < 0 || (ncalls > 0 && !calls)) { set_error("null or negative argument"); return EWF_EINVAL; }
        for (int32_t i = 0; i < ncalls; i++) {
            const ewf_call &c = calls[i];
            ewf_status st = ewf_run(c.exec, c.in, c.nin, c.scalars, c.nscalars, c.out, c.nout, c.workspace, c.workspace_bytes,
                                    c.hip_stream);
            if (st != EWF_OK) {
                if (failed) *failed = i;
                return st;
            }
        }
        return EWF_OK;
    });
}

static void fill_plan_info(const Plan *p, ewf_plan_info *info);

ewf_status ewf_debug_plan_info(ewf_exec *e, ewf_plan_info *info)
{
    return guarded([&]() -> ewf_status {
        if (!e || !info) { set_error("null argument"); return EWF_EINVAL; }
        const Plan *p = e->e.last;
        if (!p) { set_error("no plan yet"); return EWF_EINVAL; }
        fill_plan_info(p, info);
        return EWF_OK;
    });
}

static const Plan *stage_plan(ewf_exec *e, int32_t stage)
{
    if (!e || !e->e.last || stage < 0 || stage >= (int32_t)e->e.last->stages.size()) return nullptr;
    return e->e.last->stages[stage].exec->last;
}

ewf_status ewf_debug_stage_plan_info(ewf_exec *e, int32_t stage, ewf_plan_info *info)
{
    return guarded([&]() -> ewf_status {
        const Plan *p = stage_plan(e, stage);
        if (!p || !info) { set_error("no such stage"); return EWF_EINVAL; }
        fill_plan_info(p, info);
        return EWF_OK;
    });
}

const char *ewf_debug_stage_source(ewf_exec *e, int32_t stage)
{
    const Plan *p = stage_plan(e, stage);
    return p ? p->source.c_str() : "";
}

static void fill_plan_info(const Plan *p, ewf_plan_info *info)
{
    memset(info, 0, sizeof *info);
    info->kernel_class = (int)p->kclass;
    info->rank = p->canon.rank;
    for (int d = 0; d < p->canon.rank; d++) {
        info->extent[d] = p->canon.extent[d];
        info->reduced[d] = p->canon.reduced[d];
        info->tile[d] = p->tile[d];
    }
    info->vec = p->canon.vec;
    info->index_bits = p->canon.idx64 ? 64 : 32;
    info->noperands = (int)p->canon.ops.size();
    info->block_threads = p->block;
    info->grid_blocks = (int)p->grid;
    info->lds_bytes = p->lds_bytes;
    info->staged_operands = p->staged;
}

ewf_status ewf_debug_operand_strides(ewf_exec *e, int32_t k, int64_t *strides_out)
{
    return guarded([&]() -> ewf_status {
        if (!e || !strides_out) { set_error("null argument"); return EWF_EINVAL; }
        const Plan *p = e->e.last;
        if (!p || k < 0 || k >= (int)p->canon.ops.size()) { set_error("no such operand"); return EWF_EINVAL; }
        for (int d = 0; d < p->canon.rank; d++) strides_out[d] = p->canon.ops[k].stride[d];
        return EWF_OK;
    });
}

const char *ewf_debug_source(ewf_exec *e)
{
    if (!e || !e->e.last) return "";
    return e->e.last->source.c_str();
}

int32_t ewf_debug_compile_count(ewf_exec *e) { return e ? e->e.compile_count : 0; }

ewf_status ewf_debug_graph_size(ewf_exec *e, int32_t *nodes_described, int32_t *nodes_compiled)
{
    return guarded([&]() -> ewf_status {
        if (!e || !nodes_described || !nodes_compiled) { set_error("null argument"); return EWF_EINVAL; }
        *nodes_described = e->e.nodes_before;
        *nodes_compiled = e->e.nodes_after;
        return EWF_OK;
    });
}

ewf_status ewf_set_cache_dir(const char *path)
{
    return guarded([&]() -> ewf_status {
        set_cache_dir(path);
        return EWF_OK;
    });
}

ewf_status ewf_debug_cache_stats(int32_t *memory_hits, int32_t *disk_hits, int32_t *compiles)
{
    return guarded([&]() -> ewf_status {
        if (!memory_hits || !disk_hits || !compiles) { set_error("null argument"); return EWF_EINVAL; }
        int a, b, c;
        cache_stats(&a, &b, &c);
        *memory_hits = a; *disk_hits = b; *compiles = c;
        return EWF_OK;
    });
}

ewf_status ewf_debug_inject_fault(int32_t kind, int32_t after)
{
    if (kind < 0 || kind > 2 || after < 0) { set_error("bad argument"); return EWF_EINVAL; }
    arm_fault(kind, after);
    return EWF_OK;
}

ewf_status ewf_debug_peak_concurrent_compiles(int32_t *peak)
{
    if (!peak) { set_error("null argument"); return EWF_EINVAL; }
    *peak = peak_concurrent_compiles();
    return EWF_OK;
}

ewf_status ewf_copy_bytes(void *dst, const void *src, size_t nbytes, void *hip_stream)
{
    return guarded([&]() -> ewf_status {
        if (nbytes == 0) return EWF_OK;
        if (!dst || !src || (nbytes & 15) || ((uintptr_t)dst & 15) || ((uintptr_t)src & 15)) {
            set_error("copy needs 16-byte aligned pointers and a multiple of 16 bytes");
            return EWF_EINVAL;
        }
        aux_copy(dst, src, nbytes, (hipStream_t)hip_stream);
        hipError_t he = hipGetLastError();
        if (he != hipSuccess) { set_error("copy launch: %s", hipGetErrorString(he)); return EWF_EHIP; }
        return EWF_OK;
    });
}

}  // extern "C"
