// Typed scalar graph: construction, type/broadcast inference and the reduce structure
// (paper section 2.1.1: variables are typed by data type, rank and broadcastable pattern;
// apply nodes are in static-single-assignment form).
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <stdexcept>

#include "ewf_internal.h"

namespace ewf {

static thread_local std::string g_error;
static thread_local const char *g_static_error = nullptr;   // a message that needed no memory (takes precedence)

void set_error(const char *fmt, ...)
{
    char buf[4096];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_static_error = nullptr;
    g_error = buf;
}

void set_error_str(const std::string &s) { g_static_error = nullptr; g_error = s; }
void set_error_static(const char *text) noexcept { g_static_error = text; }
const char *get_error() { return g_static_error ? g_static_error : g_error.c_str(); }

// fault injection for tests of the ABI's exception barrier: 0 off, 1 std::bad_alloc, 2 std::runtime_error
static thread_local int g_fault_kind = 0, g_fault_after = 0;

void arm_fault(int kind, int after) { g_fault_kind = kind; g_fault_after = after; }

void fault_point()
{
    if (g_fault_kind == 0) return;
    if (g_fault_after-- > 0) return;
    const int kind = g_fault_kind;
    g_fault_kind = 0;
    if (kind == 1) throw std::bad_alloc();
    throw std::runtime_error("injected fault");
}

uint32_t all_mask(int ndim) { return ndim >= 32 ? 0xffffffffu : ((1u << ndim) - 1u); }

static bool is_value_type(int t) { return t == EWF_F32 || t == EWF_I32; }

// Fills vtype / bcast / dropped / depth of node n from its arguments.  Returns a status.
static ewf_status infer_node(Graph &g, int n)
{
    Node &nd = g.nodes[n];
    const uint32_t all = all_mask(g.ndim);
    for (int a = 0; a < nd.nargs; a++) {
        if (nd.args[a] < 0 || nd.args[a] >= n) {
            set_error("argument %d of node %d is not an earlier value", a, n);
            return EWF_EINVAL;
        }
    }
    auto arg = [&](int a) -> const Node & { return g.nodes[nd.args[a]]; };
    nd.depth = 0;
    for (int a = 0; a < nd.nargs; a++) nd.depth = std::max(nd.depth, arg(a).depth);
    switch (nd.kind) {
    case NodeKind::Input:
        nd.vtype = (nd.storage == EWF_I32) ? EWF_I32 : EWF_F32;
        nd.bcast &= all;
        nd.dropped = nd.in_dropped & nd.bcast;
        return EWF_OK;
    case NodeKind::Scalar:
    case NodeKind::Const:
        nd.bcast = all;
        nd.dropped = 0;
        return EWF_OK;
    case NodeKind::Iota:
        nd.vtype = EWF_I32;
        nd.bcast = all & ~(1u << nd.index);
        nd.dropped = 0;
        return EWF_OK;
    case NodeKind::Cast:
        nd.vtype = (nd.op == EWF_I32) ? EWF_I32 : EWF_F32;
        nd.bcast = arg(0).bcast;
        nd.dropped = arg(0).dropped;
        return EWF_OK;
    case NodeKind::Reduce: {
        if (nd.axes == 0 || (nd.axes & ~all)) {
            set_error("reduce node %d: bad axes", n);
            return EWF_EINVAL;
        }
        nd.vtype = (nd.op == EWF_RARGMAX) ? EWF_I32 : arg(0).vtype;
        nd.bcast = arg(0).bcast | nd.axes;
        nd.dropped = (arg(0).dropped | (nd.keep ? 0u : nd.axes)) & nd.bcast;
        nd.depth = arg(0).depth + 1;
        return EWF_OK;
    }
    case NodeKind::Apply: {
        uint32_t bc = all, dr = 0;
        for (int a = 0; a < nd.nargs; a++) { bc &= arg(a).bcast; dr |= arg(a).dropped; }
        nd.bcast = bc;
        nd.dropped = dr & bc;
        auto need = [&](int k) {
            if (nd.nargs != k) { set_error("operation %d takes %d argument(s)", nd.op, k); return false; }
            return true;
        };
        auto same = [&](int a, int b) {
            if (arg(a).vtype != arg(b).vtype) {
                set_error("node %d: operands have different value types (insert a cast)", n);
                return false;
            }
            return true;
        };
        auto real = [&](int a) {
            if (arg(a).vtype != EWF_F32) { set_error("node %d: operation needs float32 operands", n); return false; }
            return true;
        };
        switch (nd.op) {
        case EWF_ADD: case EWF_SUB: case EWF_MUL: case EWF_MAX: case EWF_MIN:
            if (!need(2)) return EWF_EINVAL;
            if (!same(0, 1)) return EWF_ETYPE;
            nd.vtype = arg(0).vtype; return EWF_OK;
        case EWF_NEG: case EWF_ABS: case EWF_SQR:
            if (!need(1)) return EWF_EINVAL;
            nd.vtype = arg(0).vtype; return EWF_OK;
        case EWF_DIV: case EWF_POW:
            if (!need(2)) return EWF_EINVAL;
            if (!real(0) || !real(1)) return EWF_ETYPE;
            nd.vtype = EWF_F32; return EWF_OK;
        case EWF_EXP: case EWF_LOG: case EWF_LOG1P: case EWF_SQRT: case EWF_TANH: case EWF_SIGMOID:
        case EWF_EXPM1: case EWF_RECIP:
            if (!need(1)) return EWF_EINVAL;
            if (!real(0)) return EWF_ETYPE;
            nd.vtype = EWF_F32; return EWF_OK;
        case EWF_GT: case EWF_GE: case EWF_LT: case EWF_LE: case EWF_EQ: case EWF_NE:
            if (!need(2)) return EWF_EINVAL;
            if (!same(0, 1)) return EWF_ETYPE;
            nd.vtype = EWF_I32; return EWF_OK;
        case EWF_WHERE:
            if (!need(3)) return EWF_EINVAL;
            if (!same(1, 2)) return EWF_ETYPE;
            nd.vtype = arg(1).vtype; return EWF_OK;
        default:
            set_error("unknown operation %d", nd.op);
            return EWF_EINVAL;
        }
    }
    }
    return EWF_EINVAL;
}

static ewf_value push_node(Graph *g, Node nd)
{
    if (!g) { set_error("null graph"); return EWF_EINVAL; }
    if (g->nodes.size() >= 4096) { set_error("graph too large"); return EWF_EINVAL; }
    fault_point();
    g->nodes.push_back(nd);
    int id = (int)g->nodes.size() - 1;
    ewf_status st = infer_node(*g, id);
    if (st != EWF_OK) { g->nodes.pop_back(); return st; }
    return id;
}

ewf_status finalize_graph(Graph &g)
{
    for (int n = 0; n < (int)g.nodes.size(); n++) {
        ewf_status st = infer_node(g, n);
        if (st != EWF_OK) return st;
    }
    if (g.outputs.empty()) { set_error("graph has no output"); return EWF_EINVAL; }
    for (const OutputDecl &o : g.outputs) {
        const Node &v = g.nodes[o.value];
        bool want_int = (o.storage == EWF_I32);
        if ((v.vtype == EWF_I32) != want_int) {
            set_error("output of value %d: storage type does not match the value type (insert a cast)", o.value);
            return EWF_ETYPE;
        }
    }
    return EWF_OK;
}

ReduceInfo analyse_reductions(const Graph &g, uint32_t unit_mask)
{
    ReduceInfo r;
    const int N = (int)g.nodes.size();
    r.edepth.assign(N, 0);
    // which nodes matter for the outputs
    std::vector<char> live(N, 0);
    for (const OutputDecl &o : g.outputs) live[o.value] = 1;
    for (int n = N - 1; n >= 0; n--)
        if (live[n]) for (int a = 0; a < g.nodes[n].nargs; a++) live[g.nodes[n].args[a]] = 1;

    // axes along which a reduce node's argument really varies in this call
    auto effective = [&](const Node &nd) { return nd.axes & ~g.nodes[nd.args[0]].bcast & ~unit_mask; };

    for (int n = 0; n < N; n++) {
        const Node &nd = g.nodes[n];
        for (int a = 0; a < nd.nargs; a++) r.edepth[n] = std::max(r.edepth[n], r.edepth[nd.args[a]]);
        if (nd.kind == NodeKind::Reduce && effective(nd)) r.edepth[n]++;
    }
    // first-level reductions define the fused axes
    for (int n = 0; n < N; n++) {
        const Node &nd = g.nodes[n];
        if (!live[n] || nd.kind != NodeKind::Reduce) continue;
        uint32_t eff = effective(nd);
        if (eff == 0) continue;                         // reduction over extent-1 axes: identity
        r.has_reduce = true;
        if (r.edepth[nd.args[0]] == 0 && r.axes == 0) r.axes = eff;
    }
    if (!r.has_reduce) return r;
    if (r.axes == 0) { r.unsupported = "no first-level reduction"; return r; }

    std::vector<char> after_cross(N, 0);                // depends on a cross reduction
    for (int n = 0; n < N; n++) {
        const Node &nd = g.nodes[n];
        if (!live[n]) continue;
        for (int a = 0; a < nd.nargs; a++) if (after_cross[nd.args[a]]) after_cross[n] = 1;
        if (nd.kind != NodeKind::Reduce) continue;
        uint32_t eff = effective(nd);
        if (eff == 0) continue;
        const Node &arg = g.nodes[nd.args[0]];
        if (after_cross[n]) { r.unsupported = "reduction of a value that depends on a cross-group reduction"; return r; }
        if (eff == r.axes) {
            r.level_nodes.push_back(n);
            r.max_depth = std::max(r.max_depth, r.edepth[n]);
        } else if ((eff & r.axes) == 0 && ((arg.bcast | unit_mask) & r.axes) == r.axes) {
            // reduces per-group values over kept axes
            if (r.cross_axes && r.cross_axes != eff) { r.unsupported = "cross-group reductions over different axes"; return r; }
            r.cross_axes = eff;
            r.cross_nodes.push_back(n);
            after_cross[n] = 1;
        } else {
            r.unsupported = "reductions over different axis sets in one expression";
            return r;
        }
    }
    // what is computed from a cross-group reduction exists once: everything else it uses
    // must be constant over the iteration space
    const uint32_t all = all_mask(g.ndim);
    for (int n = 0; n < N; n++) {
        if (!live[n] || !after_cross[n]) continue;
        const Node &nd = g.nodes[n];
        if (nd.kind == NodeKind::Reduce) continue;
        for (int a = 0; a < nd.nargs; a++) {
            const Node &arg = g.nodes[nd.args[a]];
            if (!after_cross[nd.args[a]] && ((arg.bcast | unit_mask) & all) != all) {
                r.unsupported = "a value combines a cross-group reduction with something that varies";
                return r;
            }
        }
    }
    return r;
}

}  // namespace ewf

// =========================================================================================
// C ABI: graph construction

using namespace ewf;

struct ewf_graph { Graph g; };

extern "C" {

ewf_status ewf_graph_create(int32_t ndim, ewf_graph **out)
{
    return guarded([&]() -> ewf_status {
        if (!out || ndim < 0 || ndim > EWF_MAX_DIMS) { set_error("bad rank"); return EWF_EINVAL; }
        ewf_graph *g = new (std::nothrow) ewf_graph();
        if (!g) return EWF_ENOMEM;
        g->g.ndim = ndim;
        *out = g;
        return EWF_OK;
    });
}

void ewf_graph_destroy(ewf_graph *g) { delete g; }

ewf_value ewf_input(ewf_graph *g, ewf_dtype storage, const uint8_t *bcast_flags)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (storage != EWF_F32 && storage != EWF_F16 && storage != EWF_I32) { set_error("bad storage type"); return EWF_ETYPE; }
        if (g->g.ndim > 0 && !bcast_flags) { set_error("null broadcast pattern"); return EWF_EINVAL; }
        Node nd;
        nd.kind = NodeKind::Input;
        nd.storage = storage;
        nd.index = g->g.ninputs;
        for (int d = 0; d < g->g.ndim; d++) if (bcast_flags[d]) nd.bcast |= 1u << d;
        ewf_value v = push_node(&g->g, nd);
        if (v >= 0) { g->g.ninputs++; g->g.input_node.push_back(v); }
        return v;
    });
}

ewf_value ewf_scalar(ewf_graph *g, ewf_dtype dtype)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (!is_value_type(dtype)) { set_error("scalar type must be float32 or int32"); return EWF_ETYPE; }
        Node nd;
        nd.kind = NodeKind::Scalar;
        nd.vtype = dtype;
        nd.index = g->g.nscalars;
        ewf_value v = push_node(&g->g, nd);
        if (v >= 0) { g->g.nscalars++; g->g.scalar_node.push_back(v); }
        return v;
    });
}

ewf_value ewf_const(ewf_graph *g, ewf_dtype dtype, double value)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (!is_value_type(dtype)) { set_error("literal type must be float32 or int32"); return EWF_ETYPE; }
        Node nd;
        nd.kind = NodeKind::Const;
        nd.vtype = dtype;
        nd.cval = value;
        return push_node(&g->g, nd);
    });
}

ewf_value ewf_iota(ewf_graph *g, int32_t axis)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (axis < 0 || axis >= g->g.ndim) { set_error("iota axis out of range"); return EWF_EINVAL; }
        Node nd;
        nd.kind = NodeKind::Iota;
        nd.index = axis;
        return push_node(&g->g, nd);
    });
}

ewf_value ewf_apply(ewf_graph *g, ewf_op op, const ewf_value *args, int32_t nargs)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (nargs < 1 || nargs > 3 || !args) { set_error("bad argument count"); return EWF_EINVAL; }
        if ((int)op < 0 || op >= EWF_OP_COUNT) { set_error("unknown operation"); return EWF_EINVAL; }
        Node nd;
        nd.kind = NodeKind::Apply;
        nd.op = op;
        nd.nargs = nargs;
        for (int a = 0; a < nargs; a++) nd.args[a] = args[a];
        return push_node(&g->g, nd);
    });
}

ewf_value ewf_cast(ewf_graph *g, ewf_value v, ewf_dtype to)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (to != EWF_F32 && to != EWF_F16 && to != EWF_I32) { set_error("bad cast target"); return EWF_ETYPE; }
        Node nd;
        nd.kind = NodeKind::Cast;
        nd.op = to;
        nd.nargs = 1;
        nd.args[0] = v;
        return push_node(&g->g, nd);
    });
}

ewf_value ewf_reduce(ewf_graph *g, ewf_redop op, ewf_value v, const int32_t *axes, int32_t naxes,
                     int32_t keep_as_bcast)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if ((int)op < 0 || op > EWF_RARGMAX) { set_error("unknown reduction"); return EWF_EINVAL; }
        if (naxes < 1 || !axes) { set_error("reduce needs at least one axis"); return EWF_EINVAL; }
        Node nd;
        nd.kind = NodeKind::Reduce;
        nd.op = op;
        nd.nargs = 1;
        nd.args[0] = v;
        nd.keep = keep_as_bcast != 0;
        for (int a = 0; a < naxes; a++) {
            if (axes[a] < 0 || axes[a] >= g->g.ndim) { set_error("reduce axis out of range"); return EWF_EINVAL; }
            if (nd.axes & (1u << axes[a])) { set_error("reduce axis repeated"); return EWF_EINVAL; }
            nd.axes |= 1u << axes[a];
        }
        return push_node(&g->g, nd);
    });
}

ewf_status ewf_output(ewf_graph *g, ewf_value v, ewf_dtype storage)
{
    return guarded([&]() -> ewf_status {
        if (!g) { set_error("null graph"); return EWF_EINVAL; }
        if (v < 0 || v >= (int)g->g.nodes.size()) { set_error("output of an unknown value"); return EWF_EINVAL; }
        if (storage != EWF_F32 && storage != EWF_F16 && storage != EWF_I32) { set_error("bad storage type"); return EWF_ETYPE; }
        const Node &nd = g->g.nodes[v];
        if ((nd.vtype == EWF_I32) != (storage == EWF_I32)) {
            set_error("output storage type does not match the value type (insert a cast)");
            return EWF_ETYPE;
        }
        g->g.outputs.push_back({v, storage});
        return EWF_OK;
    });
}

const char *ewf_last_error(void) { return get_error(); }

int32_t ewf_debug_graph_count(const ewf_graph *g) { return g ? (int32_t)g->g.nodes.size() : 0; }

ewf_status ewf_debug_graph_node(const ewf_graph *g, int32_t i, ewf_node_info *info)
{
    return guarded([&]() -> ewf_status {
        if (!g || !info || i < 0 || i >= (int32_t)g->g.nodes.size()) { set_error("no such node"); return EWF_EINVAL; }
        const Node &nd = g->g.nodes[i];
        info->kind = (int32_t)nd.kind;
        info->op = nd.op;
        info->nargs = nd.nargs;
        for (int a = 0; a < 3; a++) info->args[a] = nd.args[a];
        info->index = nd.index;
        info->axes = nd.axes;
        info->keep = nd.keep ? 1 : 0;
        info->vtype = (int32_t)nd.vtype;
        info->storage = (int32_t)nd.storage;
        info->bcast = nd.bcast;
        info->cval = nd.cval;
        return EWF_OK;
    });
}

}  // extern "C"

namespace ewf {
const Graph &graph_of(const ewf_graph *g) { return g->g; }
Graph &graph_of_mut(ewf_graph *g) { return g->g; }
ewf_value graph_push(Graph *g, Node nd) { return push_node(g, nd); }
}
