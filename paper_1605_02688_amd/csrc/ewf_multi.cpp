// Plans in several passes.
//
// The single-kernel classes cover one set of reduced axes, chained reductions only along the
// innermost dimension, and outputs that use a reduction only per group.  Anything else (a value
// normalised by a column sum, reductions over unrelated axis sets in one description, a chain
// of reductions over an outer axis) is split the way the paper's fusion stage groups a graph
// into kernels (section 2.2.1): the reductions that depend on no other reduction are
// materialised by kernels of their own into temporaries inside the caller's workspace, the rest
// of the graph then reads them as broadcastable inputs, and so on until what remains fits one
// kernel.  Every stage is an ordinary sub-expression with its own executable and plan cache.
#include <algorithm>
#include <cstring>
#include <map>

#include "ewf_internal.h"

namespace ewf {

namespace {

constexpr uint64_t kFakeBase = (uint64_t)0x0F00 << 44;     // stands in for workspace addresses while planning

struct Cut { int temp; };

// Builds the sub-expression that computes `targets` (node id, storage, forced keep) from the
// caller's inputs and the temporaries of already materialised nodes.
void build_stage(const Graph &g, const std::vector<std::pair<int, ewf_dtype>> &targets, bool force_keep,
                 const std::map<int, int> &cuts, Exec &sub, std::vector<int> &in_src)
{
    const int N = (int)g.nodes.size();
    std::vector<char> need(N, 0);
    for (auto &t : targets) need[t.first] = 1;
    for (int n = N - 1; n >= 0; n--) {
        if (!need[n] || cuts.count(n)) continue;
        for (int a = 0; a < g.nodes[n].nargs; a++) need[g.nodes[n].args[a]] = 1;
    }
    Graph &h = sub.g;
    h = Graph();
    h.ndim = g.ndim;
    std::vector<int> pos(N, -1);
    // every run-time scalar keeps its ordinal
    for (int k = 0; k < g.nscalars; k++) {
        Node nd = g.nodes[g.scalar_node[k]];
        pos[g.scalar_node[k]] = (int)h.nodes.size();
        h.scalar_node.push_back((int)h.nodes.size());
        h.nodes.push_back(nd);
    }
    h.nscalars = g.nscalars;
    in_src.clear();
    for (int n = 0; n < N; n++) {
        if (!need[n] || pos[n] >= 0) continue;
        Node nd = g.nodes[n];
        auto cut = cuts.find(n);
        if (cut != cuts.end()) {
            Node in;
            in.kind = NodeKind::Input;
            in.storage = nd.vtype == EWF_I32 ? EWF_I32 : EWF_F32;
            in.bcast = nd.bcast;
            in.in_dropped = nd.dropped;
            in.index = h.ninputs++;
            in_src.push_back(-(cut->second + 1));
            pos[n] = (int)h.nodes.size();
            h.input_node.push_back(pos[n]);
            h.nodes.push_back(in);
            continue;
        }
        if (nd.kind == NodeKind::Input) {
            in_src.push_back(nd.index);
            nd.index = h.ninputs++;
            pos[n] = (int)h.nodes.size();
            h.input_node.push_back(pos[n]);
            h.nodes.push_back(nd);
            continue;
        }
        for (int a = 0; a < nd.nargs; a++) nd.args[a] = pos[nd.args[a]];
        if (force_keep && nd.kind == NodeKind::Reduce)
            for (auto &t : targets) if (t.first == n) nd.keep = true;
        pos[n] = (int)h.nodes.size();
        h.nodes.push_back(nd);
    }
    for (auto &t : targets) h.outputs.push_back({pos[t.first], t.second});
}

}  // namespace

ewf_status plan_multi(Exec &e, const Graph &g, bool strict_rows, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout, Plan &plan)
{
    const int N = (int)g.nodes.size();
    int64_t full[kMaxDims];
    ewf_status st = infer_full_extents(g, in, nin, full);
    if (st != EWF_OK) return st;
    uint32_t unit = 0;
    for (int d = 0; d < g.ndim; d++) if (full[d] == 1) unit |= 1u << d;

    std::vector<char> live(N, 0);
    for (const OutputDecl &o : g.outputs) live[o.value] = 1;
    for (int n = N - 1; n >= 0; n--)
        if (live[n]) for (int a = 0; a < g.nodes[n].nargs; a++) live[g.nodes[n].args[a]] = 1;

    plan.stages.clear();
    plan.temps.clear();
    std::map<int, int> cuts;                            // node -> temporary
    size_t ws = 0;
    auto align_up = [](size_t v) { return (v + 255) / 256 * 256; };

    // tensors of a stage while planning: the caller's, or a temporary at a stand-in address
    auto stage_tensors = [&](const Stage &sg, std::vector<ewf_tensor> &tin, std::vector<ewf_tensor> &tout) {
        tin.clear(); tout.clear();
        for (int s : sg.in_src) {
            if (s >= 0) tin.push_back(in[s]);
            else { const Temp &t = plan.temps[-s - 1]; tin.push_back({(void *)(uintptr_t)(kFakeBase + t.offset), t.shape, t.strides}); }
        }
        for (int d : sg.out_dst) {
            if (d >= 0) tout.push_back(out[d]);
            else { const Temp &t = plan.temps[-d - 1]; tout.push_back({(void *)(uintptr_t)(kFakeBase + t.offset), t.shape, t.strides}); }
        }
    };
    auto try_stage = [&](Stage &sg) -> ewf_status {
        sg.exec->opts = e.opts;
        sg.exec->math_flavour = e.math_flavour;
        sg.exec->auto_math = e.auto_math;
        sg.exec->is_stage = true;
        sg.exec->strict_rows = strict_rows;
        // only an index (iota) makes a stage depend on an axis that none of its inputs spans
        uint32_t iota_axes = 0;
        for (const Node &nd : sg.exec->g.nodes) if (nd.kind == NodeKind::Iota) iota_axes |= 1u << nd.index;
        sg.exec->has_forced_full = iota_axes != 0;
        for (int d = 0; d < kMaxDims; d++) sg.exec->forced_full[d] = (d < g.ndim && (iota_axes >> d & 1u)) ? full[d] : 1;
        ewf_status s2 = finalize_graph(sg.exec->g);
        if (s2 != EWF_OK) return s2;
        std::vector<ewf_tensor> tin, tout;
        stage_tensors(sg, tin, tout);
        Plan *sp = nullptr;
        s2 = make_plan(*sg.exec, tin.data(), (int)tin.size(), tout.data(), (int)tout.size(), &sp);
        if (s2 != EWF_OK) return s2;
        sg.ws_bytes = sp->workspace_bytes;
        return EWF_OK;
    };

    // Element-wise outputs that an earlier pass can write on its way.  A pass that materialises
    // reductions and already walks the full extents evaluates such an output from the values it
    // has in registers anyway; left to the last pass it costs one more sweep over the inputs
    // (bias + ReLU + per-channel sums on [128, 512, 28, 28]: three sweeps instead of two).
    // Only outputs that depend on no reduction, span every axis and share no memory with any
    // input qualify (an in-place output would change what later passes read).
    std::vector<char> written(nout, 0);
    auto byte_span = [&](const ewf_tensor &t, int rank, int itemsize, uint64_t &lo, uint64_t &hi) {
        int64_t below = 0, above = 0;                       // reach of the view from its pointer, in elements
        bool empty = false;
        for (int d = 0; d < rank; d++) {
            if (t.shape[d] == 0) empty = true;
            else if (t.strides[d] < 0) below += (t.shape[d] - 1) * -t.strides[d];
            else above += (t.shape[d] - 1) * t.strides[d];
        }
        lo = (uint64_t)(uintptr_t)t.ptr - (uint64_t)below * itemsize;
        hi = empty ? lo : (uint64_t)(uintptr_t)t.ptr + (uint64_t)(above + 1) * itemsize;
    };
    auto can_ride = [&](int k) {
        const OutputDecl &od = g.outputs[k];
        if (written[k] || (g.nodes[od.value].bcast & ~unit) || g.nodes[od.value].dropped) return false;
        std::vector<char> cone(N, 0);
        cone[od.value] = 1;
        for (int n = N - 1; n >= 0; n--) {
            if (!cone[n]) continue;
            if (g.nodes[n].kind == NodeKind::Reduce || cuts.count(n)) return false;
            for (int a = 0; a < g.nodes[n].nargs; a++) cone[g.nodes[n].args[a]] = 1;
        }
        uint64_t olo, ohi, ilo, ihi;
        byte_span(out[k], g.ndim, od.storage == EWF_F16 ? 2 : 4, olo, ohi);
        for (int i = 0; i < nin; i++) {
            byte_span(in[i], g.ndim, g.nodes[g.input_node[i]].storage == EWF_F16 ? 2 : 4, ilo, ihi);
            if (olo < ihi && ilo < ohi) return false;
        }
        return true;
    };

    for (int round = 0; round < 16; round++) {
        bool all_written = true;
        for (int k = 0; k < nout; k++) all_written = all_written && written[k];
        if (all_written && !plan.stages.empty()) break;
        // does what remains fit one kernel?
        {
            Stage fin;
            fin.exec.reset(new Exec());
            std::vector<std::pair<int, ewf_dtype>> targets;
            for (int k = 0; k < nout; k++) if (!written[k]) { targets.push_back({g.outputs[k].value, g.outputs[k].storage}); fin.out_dst.push_back(k); }
            build_stage(g, targets, false, cuts, *fin.exec, fin.in_src);
            st = try_stage(fin);
            if (st == EWF_OK) {
                plan.stages.push_back(std::move(fin));
                break;
            }
            if (st != EWF_EUNSUPPORTED) return st;
        }
        // materialise the reductions that depend on no other (unmaterialised) reduction,
        // one stage per set of reduced axes
        std::vector<int> depth(N, 0);
        for (int n = 0; n < N; n++) {
            if (cuts.count(n)) { depth[n] = 0; continue; }
            const Node &nd = g.nodes[n];
            for (int a = 0; a < nd.nargs; a++) depth[n] = std::max(depth[n], depth[nd.args[a]]);
            if (nd.kind == NodeKind::Reduce && (nd.axes & ~g.nodes[nd.args[0]].bcast & ~unit)) depth[n]++;
        }
        std::map<uint32_t, std::vector<int>> groups;
        for (int n = 0; n < N; n++) {
            const Node &nd = g.nodes[n];
            if (!live[n] || cuts.count(n) || nd.kind != NodeKind::Reduce || depth[n] != 1) continue;
            const uint32_t eff = nd.axes & ~g.nodes[nd.args[0]].bcast & ~unit;
            if (eff) groups[eff].push_back(n);
        }
        if (groups.empty()) { set_error("no reduction left to split off"); return EWF_EUNSUPPORTED; }
        for (auto &gr : groups) {
            // Values computed from this stage's reductions that are still constant along the reduced
            // axes (the reciprocal deviation of a normalisation: one number per column) are
            // evaluated once per group by this stage and handed on as temporaries too; a later,
            // element-wise stage would evaluate them once per element.
            std::vector<int> handed = gr.second;
            std::vector<char> glevel(N, 0), dep(N, 0);
            if (!e.opts.no_rewrite) {
                const uint32_t eff = gr.first;
                std::vector<char> mine(N, 0);
                for (int n : gr.second) mine[n] = 1;
                for (int n = 0; n < N; n++) {
                    const Node &nd = g.nodes[n];
                    if (mine[n]) { glevel[n] = dep[n] = 1; continue; }
                    if (cuts.count(n) || nd.kind == NodeKind::Input || nd.kind == NodeKind::Scalar || nd.kind == NodeKind::Const ||
                        nd.kind == NodeKind::Iota) { glevel[n] = ((nd.bcast | unit) & eff) == eff; continue; }
                    if (nd.kind == NodeKind::Reduce) continue;
                    bool all = nd.nargs > 0, any = false;
                    for (int a = 0; a < nd.nargs; a++) { all = all && glevel[nd.args[a]]; any = any || dep[nd.args[a]]; }
                    glevel[n] = all && any;
                    dep[n] = glevel[n];
                }
                // the outermost such values: used by something that varies along the reduced axes
                std::vector<char> used_outside(N, 0);
                for (int n = 0; n < N; n++) {
                    if (!live[n] || glevel[n]) continue;
                    for (int a = 0; a < g.nodes[n].nargs; a++) used_outside[g.nodes[n].args[a]] = 1;
                }
                for (int n = 0; n < N; n++)
                    if (live[n] && glevel[n] && dep[n] && !mine[n] && !cuts.count(n) && used_outside[n] && g.nodes[n].kind != NodeKind::Reduce)
                        handed.push_back(n);
            }
            // one attempt with a given list of values to hand on; a failed attempt leaves no trace
            // Outputs that are such values (a mean, a variance: one number per group) are written by
            // this stage as well: left to an element-wise stage, every element of the group would
            // store the same number to the same place.
            auto attempt = [&](const std::vector<int> &hand, bool group_outputs) -> ewf_status {
                const size_t ntemps = plan.temps.size(), ws0 = ws;
                Stage sg;
                sg.exec.reset(new Exec());
                std::vector<std::pair<int, ewf_dtype>> targets;
                for (int n : hand) targets.push_back({n, g.nodes[n].vtype == EWF_I32 ? EWF_I32 : EWF_F32});
                build_stage(g, targets, true, cuts, *sg.exec, sg.in_src);
                for (int n : hand) {
                    Temp t;
                    t.dtype = g.nodes[n].vtype == EWF_I32 ? EWF_I32 : EWF_F32;
                    int64_t count = 1;
                    for (int d = g.ndim - 1; d >= 0; d--) {
                        t.shape[d] = (g.nodes[n].bcast & (1u << d)) ? 1 : full[d];
                        t.strides[d] = count;
                        count *= t.shape[d];
                    }
                    t.bytes = (size_t)count * 4;
                    t.offset = ws;
                    ws = align_up(ws + t.bytes);
                    plan.temps.push_back(t);
                    sg.out_dst.push_back(-(int)plan.temps.size());
                }
                std::vector<int> gouts;
                if (group_outputs)
                    for (int k = 0; k < nout; k++) {
                        const int v = g.outputs[k].value;
                        if (!written[k] && glevel[v] && dep[v] && !g.nodes[v].dropped) gouts.push_back(k);
                    }
                if (!gouts.empty()) {
                    for (int k : gouts) { targets.push_back({g.outputs[k].value, g.outputs[k].storage}); sg.out_dst.push_back(k); }
                    build_stage(g, targets, true, cuts, *sg.exec, sg.in_src);
                }
                // does this pass walk the full extents (then element-wise outputs can ride along)?
                bool spans_all = true;
                for (int d = 0; d < g.ndim && spans_all; d++) {
                    if (full[d] <= 1) continue;
                    bool some = false;
                    for (int node : sg.exec->g.input_node) if (!(sg.exec->g.nodes[node].bcast >> d & 1u)) some = true;
                    spans_all = some;
                }
                std::vector<int> riders;
                if (spans_all && !e.opts.no_rewrite)
                    for (int k = 0; k < nout; k++) if (can_ride(k)) riders.push_back(k);
                bool done = false;
                if (!riders.empty()) {
                    Stage both;
                    both.exec.reset(new Exec());
                    std::vector<std::pair<int, ewf_dtype>> all = targets;
                    for (int k : riders) all.push_back({g.outputs[k].value, g.outputs[k].storage});
                    build_stage(g, all, true, cuts, *both.exec, both.in_src);
                    both.out_dst = sg.out_dst;
                    for (int k : riders) both.out_dst.push_back(k);
                    if (try_stage(both) == EWF_OK) {
                        for (int k : riders) written[k] = 1;
                        sg = std::move(both);
                        done = true;
                    }
                }
                if (!done) {
                    const ewf_status s3 = try_stage(sg);
                    if (s3 != EWF_OK) { plan.temps.resize(ntemps); ws = ws0; return s3; }
                }
                for (int k : gouts) written[k] = 1;
                for (size_t i = 0; i < hand.size(); i++) cuts[hand[i]] = (int)plan.temps.size() - (int)hand.size() + (int)i;
                plan.stages.push_back(std::move(sg));
                return EWF_OK;
            };
            st = attempt(handed, !e.opts.no_rewrite);
            if (st != EWF_OK && !e.opts.no_rewrite) st = attempt(gr.second, false);
            if (st != EWF_OK) return st;
        }
        if (round == 15) { set_error("too many reduction levels"); return EWF_EUNSUPPORTED; }
    }
    // A caller's input that a later stage reads again: the earlier stage is planned once more
    // knowing that (its loads of that tensor then leave it in the memory-side cache, see the
    // streaming hint of the canonical layout).
    for (size_t i = 0; i + 1 < plan.stages.size(); i++) {
        Stage &sg = plan.stages[i];
        std::vector<char> again(sg.in_src.size(), 0);
        bool any = false;
        for (size_t a = 0; a < sg.in_src.size(); a++) {
            if (sg.in_src[a] < 0) continue;
            for (size_t j = i + 1; j < plan.stages.size(); j++)
                if (std::find(plan.stages[j].in_src.begin(), plan.stages[j].in_src.end(), sg.in_src[a]) != plan.stages[j].in_src.end()) again[a] = 1;
            any = any || again[a];
        }
        if (!any || e.opts.streaming != 0) continue;
        sg.exec->read_again = again;
        sg.exec->plans.clear();
        sg.exec->last = nullptr;
        if (try_stage(sg) != EWF_OK) {
            sg.exec->read_again.clear();
            sg.exec->plans.clear();
            sg.exec->last = nullptr;
            st = try_stage(sg);
            if (st != EWF_OK) return st;
        }
    }
    for (Stage &sg : plan.stages) {
        sg.ws_offset = ws;
        ws = align_up(ws + sg.ws_bytes);
    }
    plan.workspace_bytes = ws;
    plan.finish_grid = 0;
    plan.grid = (int64_t)plan.stages.size();
    return EWF_OK;
}

ewf_status plan_empty_rest(Exec &e, const int64_t *full, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout,
                           const std::vector<int> &outs, Plan &plan)
{
    (void)nin; (void)nout;
    const Graph &g = e.g;
    const int N = (int)g.nodes.size();
    auto align_up = [](size_t v) { return (v + 255) / 256 * 256; };
    std::vector<char> need(N, 0);
    for (int k : outs) need[g.outputs[k].value] = 1;
    std::map<int, int> cuts;
    size_t ws = 0;
    for (int n = N - 1; n >= 0; n--) {
        if (!need[n]) continue;
        const Node &nd = g.nodes[n];
        bool over_empty = false;
        if (nd.kind == NodeKind::Reduce)
            for (int d = 0; d < g.ndim; d++)
                if ((nd.axes >> d & 1u) && full[d] == 0 && !(g.nodes[nd.args[0]].bcast >> d & 1u)) over_empty = true;
        if (!over_empty) {
            for (int a = 0; a < nd.nargs; a++) need[nd.args[a]] = 1;
            continue;
        }
        if (nd.op != EWF_RSUM && nd.op != EWF_RPROD) {
            set_error("a value is computed from a maximum, minimum or arg-max over an empty axis: only sums (0) and products (1) are defined there");
            return EWF_ESHAPE;
        }
        Temp t;
        t.dtype = nd.vtype == EWF_I32 ? EWF_I32 : EWF_F32;
        int64_t count = 1;
        for (int d = g.ndim - 1; d >= 0; d--) {
            t.shape[d] = (nd.bcast >> d & 1u) ? 1 : full[d];
            t.strides[d] = count;
            count *= t.shape[d];
        }
        if (count <= 0) { set_error("internal: an empty value under an output that is not"); return EWF_ESHAPE; }
        t.bytes = (size_t)count * 4;
        t.offset = ws;
        ws = align_up(ws + t.bytes);
        plan.temps.push_back(t);
        cuts[n] = (int)plan.temps.size() - 1;
        const uint32_t one = t.dtype == EWF_I32 ? 1u : 0x3f800000u;
        plan.temp_fills.push_back({(int)plan.temps.size() - 1, nd.op == EWF_RPROD ? one : 0u});
    }
    Stage sg;
    sg.exec.reset(new Exec());
    std::vector<std::pair<int, ewf_dtype>> targets;
    for (int k : outs) { targets.push_back({g.outputs[k].value, g.outputs[k].storage}); sg.out_dst.push_back(k); }
    build_stage(g, targets, false, cuts, *sg.exec, sg.in_src);
    sg.exec->opts = e.opts;
    sg.exec->math_flavour = e.math_flavour;
    sg.exec->auto_math = e.auto_math;
    sg.exec->is_stage = true;
    uint32_t iota_axes = 0;
    for (const Node &nd : sg.exec->g.nodes) if (nd.kind == NodeKind::Iota) iota_axes |= 1u << nd.index;
    sg.exec->has_forced_full = iota_axes != 0;
    for (int d = 0; d < kMaxDims; d++) sg.exec->forced_full[d] = (d < g.ndim && (iota_axes >> d & 1u)) ? full[d] : 1;
    ewf_status st = finalize_graph(sg.exec->g);
    if (st != EWF_OK) return st;
    std::vector<ewf_tensor> tin, tout;
    for (int s : sg.in_src) {
        if (s >= 0) tin.push_back(in[s]);
        else { const Temp &t = plan.temps[-s - 1]; tin.push_back({(void *)(uintptr_t)(kFakeBase + t.offset), t.shape, t.strides}); }
    }
    for (int d : sg.out_dst) tout.push_back(out[d]);
    Plan *sp = nullptr;
    st = make_plan(*sg.exec, tin.data(), (int)tin.size(), tout.data(), (int)tout.size(), &sp);
    if (st != EWF_OK) return st;
    sg.ws_bytes = sp->workspace_bytes;
    sg.ws_offset = ws;
    ws = align_up(ws + sg.ws_bytes);
    plan.stages.push_back(std::move(sg));
    plan.workspace_bytes = ws;
    return EWF_OK;
}

ewf_status run_multi(Exec &x, Plan &p, const ewf_tensor *in, int, const double *scalars, int nscalars,
                     const ewf_tensor *out, int, void *workspace, size_t, void *hip_stream, bool no_setup)
{
    char *base = (char *)workspace;
    std::vector<ewf_tensor> tin, tout;
    for (Stage &sg : p.stages) {
        tin.clear(); tout.clear();
        for (int s : sg.in_src) {
            if (s >= 0) tin.push_back(in[s]);
            else { const Temp &t = p.temps[-s - 1]; tin.push_back({base + t.offset, t.shape, t.strides}); }
        }
        for (int d : sg.out_dst) {
            if (d >= 0) tout.push_back(out[d]);
            else { const Temp &t = p.temps[-d - 1]; tout.push_back({base + t.offset, t.shape, t.strides}); }
        }
        sg.exec->timing = x.timing;                 // timed runs record every stage's main kernel
        ewf_status st = run_exec(*sg.exec, tin.data(), (int)tin.size(), scalars, nscalars, tout.data(), (int)tout.size(),
                                 sg.ws_bytes ? base + sg.ws_offset : nullptr, sg.ws_bytes, hip_stream, no_setup);
        if (st != EWF_OK) return st;
    }
    return EWF_OK;
}

}  // namespace ewf
