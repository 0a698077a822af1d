// Rewrites of the scalar graph before code generation: the paper's canonicalisation and
// stabilisation stages (section 2.2.1: duplicates are merged, constant expressions folded,
// x * x style patterns simplified, log(1 + x) replaced by the stable log1p(x)), restricted
// to the scalar operations of one fused expression.  Every rewrite keeps the value's type,
// broadcast pattern and dropped axes, so output shapes never change.
#include <cmath>
#include <cstring>
#include <functional>
#include <map>
#include <tuple>

#include "ewf_internal.h"

namespace ewf {

namespace {

bool is_const(const Graph &g, int n, double v)
{
    const Node &nd = g.nodes[n];
    if (nd.kind != NodeKind::Const) return false;
    if (nd.vtype == EWF_I32) return (double)(int32_t)(int64_t)nd.cval == v;
    return (double)(float)nd.cval == v && !(v == 0.0 && std::signbit((float)nd.cval));
}

int32_t wrap_i32(int64_t v) { return (int32_t)(uint32_t)(uint64_t)v; }

// Value of an operation on literal arguments, in the arithmetic the kernels use (float32
// routines, wrap-around int32).  Returns false when the operation is left alone.
bool fold(const Graph &g, const Node &nd, double &out)
{
    double a[3] = {0, 0, 0};
    for (int i = 0; i < nd.nargs; i++) {
        const Node &x = g.nodes[nd.args[i]];
        if (x.kind != NodeKind::Const) return false;
        a[i] = x.vtype == EWF_I32 ? (double)(int32_t)(int64_t)x.cval : (double)(float)x.cval;
    }
    const bool isint = nd.nargs > 0 && g.nodes[nd.args[0]].vtype == EWF_I32;
    if (nd.kind == NodeKind::Cast) {
        if (nd.op == EWF_F32) { out = (double)(float)a[0]; return true; }
        if (nd.op == EWF_I32) {
            if (isint) { out = a[0]; return true; }
            float f = (float)a[0];
            out = std::isnan(f) ? 0.0 : f >= 2147483648.0f ? 2147483647.0 : f <= -2147483648.0f ? -2147483648.0 : (double)(int32_t)f;
            return true;
        }
        return false;                                   // rounding to float16: left to the kernel
    }
    if (nd.kind != NodeKind::Apply) return false;
    if (isint) {
        const int64_t x = (int64_t)a[0], y = (int64_t)a[1];
        switch (nd.op) {
        case EWF_ADD: out = wrap_i32(x + y); return true;
        case EWF_SUB: out = wrap_i32(x - y); return true;
        case EWF_MUL: out = wrap_i32((int64_t)((uint64_t)x * (uint64_t)y)); return true;
        case EWF_SQR: out = wrap_i32((int64_t)((uint64_t)x * (uint64_t)x)); return true;
        case EWF_NEG: out = wrap_i32(-x); return true;
        case EWF_ABS: out = wrap_i32(x < 0 ? -x : x); return true;
        case EWF_MAX: out = (double)(x > y ? x : y); return true;
        case EWF_MIN: out = (double)(x < y ? x : y); return true;
        case EWF_GT: out = x > y; return true;
        case EWF_GE: out = x >= y; return true;
        case EWF_LT: out = x < y; return true;
        case EWF_LE: out = x <= y; return true;
        case EWF_EQ: out = x == y; return true;
        case EWF_NE: out = x != y; return true;
        case EWF_WHERE: out = x != 0 ? a[1] : a[2]; return true;
        default: return false;
        }
    }
    const float x = (float)a[0], y = (float)a[1];
    float r;
    switch (nd.op) {
    case EWF_ADD: r = x + y; break;
    case EWF_SUB: r = x - y; break;
    case EWF_MUL: r = x * y; break;
    case EWF_DIV: r = x / y; break;
    case EWF_NEG: r = -x; break;
    case EWF_ABS: r = std::fabs(x); break;
    case EWF_SQR: r = x * x; break;
    case EWF_SQRT: r = std::sqrt(x); break;
    case EWF_EXP: r = std::exp(x); break;
    case EWF_LOG: r = std::log(x); break;
    case EWF_LOG1P: r = std::log1p(x); break;
    case EWF_EXPM1: r = std::expm1(x); break;
    case EWF_TANH: r = std::tanh(x); break;
    case EWF_SIGMOID: r = 1.0f / (1.0f + std::exp(-x)); break;
    case EWF_RECIP: r = 1.0f / x; break;
    case EWF_POW: r = std::pow(x, y); break;
    case EWF_MAX: r = (x > y || x != x) ? x : y; break;
    case EWF_MIN: r = (x < y || x != x) ? x : y; break;
    case EWF_GT: out = x > y; return true;
    case EWF_GE: out = x >= y; return true;
    case EWF_LT: out = x < y; return true;
    case EWF_LE: out = x <= y; return true;
    case EWF_EQ: out = x == y; return true;
    case EWF_NE: out = x != y; return true;
    case EWF_WHERE: out = x != 0.0f ? a[1] : a[2]; return true;
    default: return false;
    }
    if (std::isnan(r)) return false;                    // a NaN literal has no decimal form worth keeping
    out = (double)r;
    return true;
}

bool commutative(int op)
{
    return op == EWF_ADD || op == EWF_MUL || op == EWF_MAX || op == EWF_MIN || op == EWF_EQ || op == EWF_NE;
}

}  // namespace

// Rewrites `g` in place.  Returns the number of nodes removed or replaced (for tests).
int fuse_shifted_exp_sums(Graph &g, bool unless_argmax)
{
    int count = 0;
    for (Node &s : g.nodes) {
        if (s.kind != NodeKind::Reduce || s.op != EWF_RSUM || s.vtype != EWF_F32) continue;
        const Node &ex = g.nodes[s.args[0]];
        if (ex.kind != NodeKind::Apply || ex.op != EWF_EXP) continue;
        const Node &sub = g.nodes[ex.args[0]];
        if (sub.kind != NodeKind::Apply || sub.op != EWF_SUB) continue;
        const int x = sub.args[0];
        const Node &m = g.nodes[sub.args[1]];
        if (m.kind != NodeKind::Reduce || m.op != EWF_RMAX || m.args[0] != x || m.axes != s.axes) continue;
        if (g.nodes[x].vtype != EWF_F32 || g.nodes[x].bcast != ex.bcast) continue;
        if (unless_argmax) {
            bool keyed = false;
            for (const Node &o2 : g.nodes)
                if (o2.kind == NodeKind::Reduce && o2.op == EWF_RARGMAX && o2.args[0] == x && o2.axes == s.axes) keyed = true;
            if (keyed) continue;
        }
        s.op = kRSumExpShifted;
        s.args[0] = x;
        count++;
    }
    return count;
}

int fuse_centred_squares(Graph &g, const int64_t *full)
{
    int count = 0;
    for (Node &q : g.nodes) {
        if (q.kind != NodeKind::Reduce || q.op != EWF_RSUM || q.vtype != EWF_F32) continue;
        const Node &sq = g.nodes[q.args[0]];
        if (sq.kind != NodeKind::Apply) continue;
        if (!(sq.op == EWF_SQR || (sq.op == EWF_MUL && sq.args[0] == sq.args[1]))) continue;
        const Node &sub = g.nodes[sq.args[0]];
        if (sub.kind != NodeKind::Apply || sub.op != EWF_SUB) continue;
        const int x = sub.args[0];
        if (g.nodes[x].vtype != EWF_F32 || (g.nodes[x].bcast & q.axes)) continue;   // x varies along every reduced axis
        const Node &m = g.nodes[sub.args[1]];
        if (m.kind != NodeKind::Apply || (m.op != EWF_MUL && m.op != EWF_DIV)) continue;
        double n = 1.0;
        for (int d = 0; d < g.ndim; d++) if (q.axes >> d & 1u) n *= (double)full[d];
        if (n < 1.0) continue;
        int s = -1;
        for (int side = 0; side < 2 && s < 0; side++) {
            const Node &a = g.nodes[m.args[side]], &k = g.nodes[m.args[1 - side]];
            if (m.op == EWF_DIV && side == 1) break;                                // sum / n only, not n / sum
            if (a.kind != NodeKind::Reduce || a.op != EWF_RSUM || a.axes != q.axes || a.args[0] != x) continue;
            if (k.kind != NodeKind::Const || k.vtype != EWF_F32) continue;
            const float want = m.op == EWF_DIV ? (float)n : (float)(1.0 / n);
            if ((float)k.cval == want) s = m.args[side];
        }
        if (s < 0) continue;
        q.op = kRSumSqCentred;
        q.args[0] = x;
        count++;
    }
    return count;
}

int split_reduction_axes(Graph &g, uint32_t axes, uint32_t outer)
{
    if (!outer || (outer & ~axes) || outer == axes) return 0;
    Graph out;
    out.ndim = g.ndim; out.ninputs = g.ninputs; out.nscalars = g.nscalars;
    const int N = (int)g.nodes.size();
    std::vector<int> pos(N, -1);
    int count = 0;
    for (int n = 0; n < N; n++) {
        Node nd = g.nodes[n];
        for (int a = 0; a < nd.nargs; a++) nd.args[a] = pos[nd.args[a]];
        const bool splittable = nd.kind == NodeKind::Reduce && nd.axes == axes &&
                                (nd.op == EWF_RSUM || nd.op == EWF_RPROD || nd.op == EWF_RMAX || nd.op == EWF_RMIN);
        if (splittable) {
            Node first = nd;
            first.axes = outer;
            first.keep = true;
            out.nodes.push_back(first);
            nd.args[0] = (int)out.nodes.size() - 1;
            count++;
        }
        pos[n] = (int)out.nodes.size();
        out.nodes.push_back(nd);
    }
    for (int v : g.input_node) out.input_node.push_back(pos[v]);
    for (int v : g.scalar_node) out.scalar_node.push_back(pos[v]);
    for (const OutputDecl &od : g.outputs) out.outputs.push_back({pos[od.value], od.storage});
    if (finalize_graph(out) != EWF_OK) return -1;
    g = out;
    return count;
}

int rewrite_graph(Graph &g)
{
    const int N = (int)g.nodes.size();
    std::vector<int> repl(N);                           // old id -> id in `out`
    Graph out;
    out.ndim = g.ndim;
    out.ninputs = g.ninputs;
    out.nscalars = g.nscalars;
    out.input_node.assign(g.input_node.size(), -1);
    out.scalar_node.assign(g.scalar_node.size(), -1);
    int changed = 0;

    typedef std::tuple<int, int, int, int, int, int, uint64_t, uint32_t, int> Key;
    std::map<Key, int> seen;

    auto same_shape = [&](const Node &a, const Node &b) {
        return a.vtype == b.vtype && a.bcast == b.bcast && a.dropped == b.dropped;
    };
    auto push = [&](Node nd) -> int {
        // merge duplicates: same operation on the same (already merged) arguments
        if (nd.kind == NodeKind::Apply && commutative(nd.op) && nd.args[0] > nd.args[1]) std::swap(nd.args[0], nd.args[1]);
        if (nd.kind != NodeKind::Input && nd.kind != NodeKind::Scalar) {
            uint64_t bits = 0;
            if (nd.kind == NodeKind::Const) {
                if (nd.vtype == EWF_I32) bits = (uint64_t)(uint32_t)wrap_i32((int64_t)nd.cval);
                else { float f = (float)nd.cval; uint32_t b; memcpy(&b, &f, 4); bits = b; }
            }
            Key k((int)nd.kind, nd.op, nd.args[0], nd.args[1], nd.args[2], nd.kind == NodeKind::Iota ? nd.index : 0, bits,
                  nd.axes, (int)nd.vtype * 2 + (nd.keep ? 1 : 0));
            auto it = seen.find(k);
            if (it != seen.end()) { changed++; return it->second; }
            out.nodes.push_back(nd);
            seen.emplace(k, (int)out.nodes.size() - 1);
            return (int)out.nodes.size() - 1;
        }
        out.nodes.push_back(nd);
        return (int)out.nodes.size() - 1;
    };
    auto make_const = [&](ewf_dtype t, double v) {
        Node c;
        c.kind = NodeKind::Const; c.vtype = t; c.cval = v;
        c.bcast = all_mask(g.ndim);
        return push(c);
    };
    auto make_apply = [&](int op, int a0, int a1, const Node &like) {
        Node nd;
        nd.kind = NodeKind::Apply; nd.op = op; nd.nargs = a1 < 0 ? 1 : 2; nd.args[0] = a0; nd.args[1] = a1;
        nd.vtype = like.vtype; nd.bcast = like.bcast; nd.dropped = like.dropped;
        return push(nd);
    };

    // sum over axes A of (a * k), (a / k) or (-a) with k constant along A: the factor leaves the
    // sum (fewer operations per element, and the remaining sum is often one that exists already)
    std::function<int(int, uint32_t, bool)> make_sum = [&](int a, uint32_t axes, bool keep) -> int {
        const Node arg = out.nodes[a];
        auto constant_along = [&](int v) { return (out.nodes[v].bcast & axes) == axes; };
        if (arg.kind == NodeKind::Apply && arg.vtype == EWF_F32) {
            int inner = -1, factor = -1;
            if (arg.op == EWF_MUL) {
                if (constant_along(arg.args[1]) && !constant_along(arg.args[0])) { inner = arg.args[0]; factor = arg.args[1]; }
                else if (constant_along(arg.args[0]) && !constant_along(arg.args[1])) { inner = arg.args[1]; factor = arg.args[0]; }
            } else if (arg.op == EWF_DIV && constant_along(arg.args[1]) && !constant_along(arg.args[0])) {
                inner = arg.args[0]; factor = arg.args[1];
            } else if (arg.op == EWF_NEG) {
                inner = arg.args[0];
            }
            if (inner >= 0) {
                const int r = make_sum(inner, axes, keep);
                Node like = out.nodes[r];
                Node ap;
                ap.kind = NodeKind::Apply; ap.op = arg.op; ap.vtype = EWF_F32;
                ap.nargs = factor >= 0 ? 2 : 1; ap.args[0] = r; ap.args[1] = factor;
                ap.bcast = like.bcast & (factor >= 0 ? out.nodes[factor].bcast : all_mask(g.ndim));
                ap.dropped = (like.dropped | (factor >= 0 ? out.nodes[factor].dropped : 0u)) & ap.bcast;
                return push(ap);
            }
        }
        Node rd;
        rd.kind = NodeKind::Reduce; rd.op = EWF_RSUM; rd.nargs = 1; rd.args[0] = a; rd.axes = axes; rd.keep = keep;
        rd.vtype = EWF_F32;
        rd.bcast = arg.bcast | axes;
        rd.dropped = (arg.dropped | (keep ? 0u : axes)) & rd.bcast;
        rd.depth = arg.depth + 1;
        return push(rd);
    };

    for (int n = 0; n < N; n++) {
        Node nd = g.nodes[n];
        const Node orig = nd;
        for (int a = 0; a < nd.nargs; a++) nd.args[a] = repl[nd.args[a]];
        auto arg = [&](int a) -> const Node & { return out.nodes[nd.args[a]]; };
        int r = -1;

        if (nd.kind == NodeKind::Input) { r = push(nd); out.input_node[nd.index] = r; repl[n] = r; continue; }
        if (nd.kind == NodeKind::Scalar) { r = push(nd); out.scalar_node[nd.index] = r; repl[n] = r; continue; }

        // constant folding
        double cv;
        if ((nd.kind == NodeKind::Apply || nd.kind == NodeKind::Cast) && fold(out, nd, cv)) {
            repl[n] = make_const(orig.vtype, cv);
            changed++;
            continue;
        }
        if (nd.kind == NodeKind::Apply) {
            const int a0 = nd.args[0], a1 = nd.args[1];
            const bool f32 = orig.vtype == EWF_F32;
            auto keep_as = [&](int v) { if (same_shape(out.nodes[v], orig)) r = v; };
            switch (nd.op) {
            case EWF_MUL:
                if (a0 == a1) r = make_apply(EWF_SQR, a0, -1, orig);                    // x * x
                else if (is_const(out, a1, 1.0)) keep_as(a0);
                else if (is_const(out, a0, 1.0)) keep_as(a1);
                else if (f32) {
                    // (k * y) * z with k a power of two: k * (y * z), bit for bit the same (scaling by
                    // a power of two rounds nothing), and y * z is often a square or exists already;
                    // the factor then sits next to what consumes the product (exp(k * s) is one
                    // multiplication by k * log2 e and the hardware exp2)
                    for (int side = 0; side < 2 && r < 0; side++) {
                        const Node &m = out.nodes[nd.args[side]];
                        const int z = nd.args[1 - side];
                        if (m.kind != NodeKind::Apply || m.op != EWF_MUL || m.vtype != EWF_F32) continue;
                        for (int ks = 0; ks < 2 && r < 0; ks++) {
                            const Node &k = out.nodes[m.args[ks]];
                            if (k.kind != NodeKind::Const || k.vtype != EWF_F32) continue;
                            int ex = 0;
                            const float kv = (float)k.cval;
                            if (!(std::fabs(kv) >= 0x1p-20f && std::fabs(kv) <= 0x1p20f) || std::frexp(std::fabs(kv), &ex) != 0.5f) continue;
                            const int y = m.args[1 - ks];
                            Node like = orig;               // y * z varies wherever y or z does: the pattern of the whole product
                            like.bcast = out.nodes[y].bcast & out.nodes[z].bcast;
                            like.dropped = (out.nodes[y].dropped | out.nodes[z].dropped) & like.bcast;
                            if (like.bcast != orig.bcast || like.dropped != orig.dropped) continue;
                            const int inner = y == z ? make_apply(EWF_SQR, y, -1, like) : make_apply(EWF_MUL, y, z, like);
                            r = make_apply(EWF_MUL, m.args[ks], inner, orig);
                        }
                    }
                }
                break;
            case EWF_ADD:
                // x + 0 (the sum of -0 and +0 is +0; the difference cannot be seen through a
                // comparison of values, which is what every bar of this library is)
                if (is_const(out, a1, 0.0)) keep_as(a0);
                else if (is_const(out, a0, 0.0)) keep_as(a1);
                break;
            case EWF_SUB:
                if (is_const(out, a1, 0.0)) keep_as(a0);
                else if (f32 && is_const(out, a1, 1.0) && arg(0).kind == NodeKind::Apply && arg(0).op == EWF_EXP)
                    r = make_apply(EWF_EXPM1, arg(0).args[0], -1, orig);                // exp(x) - 1
                break;
            case EWF_DIV:
                if (is_const(out, a1, 1.0)) keep_as(a0);
                else if (f32 && arg(1).vtype == EWF_F32 && arg(0).vtype == EWF_F32 && (arg(1).bcast & ~arg(0).bcast) &&
                         arg(1).kind != NodeKind::Const) {
                    // a / k with k constant along an axis where a varies (a row's sum under its
                    // elements): one reciprocal per k and a product per element instead of a
                    // division per element -- about ten instructions less of the fifty that a
                    // softmax element costs.  One rounding more (1.5 units in the last place at
                    // most); a divisor below the smallest normal number overflows its reciprocal.
                    const int rk = make_apply(EWF_RECIP, a1, -1, arg(1));
                    r = make_apply(EWF_MUL, a0, rk, orig);
                }
                break;
            case EWF_NEG:
                if (arg(0).kind == NodeKind::Apply && arg(0).op == EWF_NEG) keep_as(arg(0).args[0]);
                break;
            case EWF_LOG:
                if (arg(0).kind == NodeKind::Apply && arg(0).op == EWF_ADD) {          // log(1 + x)
                    const Node &s = arg(0);
                    if (is_const(out, s.args[0], 1.0)) r = make_apply(EWF_LOG1P, s.args[1], -1, orig);
                    else if (is_const(out, s.args[1], 1.0)) r = make_apply(EWF_LOG1P, s.args[0], -1, orig);
                }
                break;
            case EWF_POW:
                if (is_const(out, a1, 2.0)) r = make_apply(EWF_SQR, a0, -1, orig);
                else if (is_const(out, a1, 1.0)) keep_as(a0);
                break;
            case EWF_WHERE:
                if (arg(0).kind == NodeKind::Const) {
                    const bool truth = arg(0).vtype == EWF_I32 ? (int32_t)(int64_t)arg(0).cval != 0 : (float)arg(0).cval != 0.0f;
                    keep_as(truth ? nd.args[1] : nd.args[2]);
                } else if (nd.args[1] == nd.args[2]) {
                    keep_as(nd.args[1]);
                }
                break;
            case EWF_MAX: case EWF_MIN:
                if (a0 == a1) keep_as(a0);
                break;
            default: break;
            }
            if (r >= 0) { repl[n] = r; changed++; continue; }
        }
        if (nd.kind == NodeKind::Reduce && nd.op == EWF_RSUM && nd.vtype == EWF_F32) {
            const int rs = make_sum(nd.args[0], nd.axes, nd.keep);
            if (same_shape(out.nodes[rs], orig)) {
                if (out.nodes[rs].kind != NodeKind::Reduce) changed++;
                repl[n] = rs;
                continue;
            }
            // (what was pushed stays as dead nodes and is removed below)
        }
        repl[n] = push(nd);
    }
    for (const OutputDecl &od : g.outputs) out.outputs.push_back({repl[od.value], od.storage});

    // drop what no output needs any more (inputs and scalars keep their places)
    const int M = (int)out.nodes.size();
    std::vector<char> live(M, 0);
    for (const OutputDecl &od : out.outputs) live[od.value] = 1;
    for (int n = M - 1; n >= 0; n--) {
        const Node &nd = out.nodes[n];
        if (nd.kind == NodeKind::Input || nd.kind == NodeKind::Scalar) live[n] = 1;
        if (live[n]) for (int a = 0; a < nd.nargs; a++) live[nd.args[a]] = 1;
    }
    std::vector<int> pos(M, -1);
    Graph fin;
    fin.ndim = out.ndim; fin.ninputs = out.ninputs; fin.nscalars = out.nscalars;
    for (int n = 0; n < M; n++) {
        if (!live[n]) { changed++; continue; }
        Node nd = out.nodes[n];
        for (int a = 0; a < nd.nargs; a++) nd.args[a] = pos[nd.args[a]];
        pos[n] = (int)fin.nodes.size();
        fin.nodes.push_back(nd);
    }
    for (int v : out.input_node) fin.input_node.push_back(pos[v]);
    for (int v : out.scalar_node) fin.scalar_node.push_back(pos[v]);
    for (const OutputDecl &od : out.outputs) fin.outputs.push_back({pos[od.value], od.storage});
    g = fin;
    return changed;
}

}  // namespace ewf
