// Reverse-mode differentiation of the scalar graph (paper section 2.1.3: gradients are
// built symbolically by walking the graph from the outputs back to the inputs, every
// operation contributing the expression of its vector-Jacobian product).  The result is more
// nodes of the same graph, so a backward pass is one more fused expression: its element-wise
// part and the sums over broadcast axes (the gradient of a bias is a column sum) run in one
// kernel like any other description.
#include <vector>

#include "ewf_internal.h"

namespace ewf {
ewf_value graph_push(Graph *g, Node nd);
Graph &graph_of_mut(ewf_graph *g);
}

using namespace ewf;

namespace {

struct Builder {
    Graph &g;
    bool failed = false;
    explicit Builder(Graph &g_) : g(g_) {}

    int push(Node nd)
    {
        if (failed) return 0;
        ewf_value v = graph_push(&g, nd);
        if (v < 0) { failed = true; return 0; }
        return v;
    }
    int lit(double v)
    {
        Node n; n.kind = NodeKind::Const; n.vtype = EWF_F32; n.cval = v;
        return push(n);
    }
    int ap(int op, int a, int b = -1, int c = -1)
    {
        Node n; n.kind = NodeKind::Apply; n.op = op;
        n.nargs = c >= 0 ? 3 : b >= 0 ? 2 : 1;
        n.args[0] = a; n.args[1] = b; n.args[2] = c;
        return push(n);
    }
    int sum_over(int v, uint32_t axes)
    {
        Node n; n.kind = NodeKind::Reduce; n.op = EWF_RSUM; n.nargs = 1; n.args[0] = v; n.axes = axes; n.keep = true;
        return push(n);
    }
    // The same value, but varying along `axes` too (one copy per index): where(iota >= 0, v, v).
    // The graph has no operation that only widens a pattern; this one keeps the value bit for bit
    // and survives the rewriter, which never changes a value's pattern.
    int expand(int v, uint32_t axes)
    {
        for (int d = 0; d < g.ndim; d++) {
            if (!(axes >> d & 1)) continue;
            Node io; io.kind = NodeKind::Iota; io.index = d;
            Node z; z.kind = NodeKind::Const; z.vtype = EWF_I32; z.cval = 0.0;
            const int everywhere = ap(EWF_GE, push(io), push(z));
            v = ap(EWF_WHERE, everywhere, v, v);
        }
        return v;
    }
};

}  // namespace

extern "C" ewf_status ewf_grad(ewf_graph *graph, const ewf_value *y, const ewf_value *ybar, int32_t ny,
                               const ewf_value *wrt, int32_t nwrt, ewf_value *grads)
{
    return guarded([&]() -> ewf_status {
        if (!graph || !y || !ybar || !wrt || !grads || ny < 1 || nwrt < 1) { set_error("null or empty argument"); return EWF_EINVAL; }
        Graph &g = graph_of_mut(graph);
        const int N = (int)g.nodes.size();
        for (int k = 0; k < ny; k++) {
            if (y[k] < 0 || y[k] >= N || ybar[k] < 0 || ybar[k] >= N) { set_error("unknown value"); return EWF_EINVAL; }
            if (g.nodes[y[k]].vtype != EWF_F32 || g.nodes[ybar[k]].vtype != EWF_F32) {
                set_error("differentiated values and their cotangents must be float32 values");
                return EWF_ETYPE;
            }
        }
        for (int j = 0; j < nwrt; j++) {
            if (wrt[j] < 0 || wrt[j] >= N) { set_error("unknown value"); return EWF_EINVAL; }
            if (g.nodes[wrt[j]].vtype != EWF_F32) { set_error("gradients are taken with respect to float32 values"); return EWF_ETYPE; }
        }

        // which nodes lie on a path from a wrt value to a differentiated value
        std::vector<char> below(N, 0), above(N, 0);
        for (int j = 0; j < nwrt; j++) below[wrt[j]] = 1;
        for (int n = 0; n < N; n++)
            for (int a = 0; a < g.nodes[n].nargs; a++) if (below[g.nodes[n].args[a]]) below[n] = 1;
        for (int k = 0; k < ny; k++) above[y[k]] = 1;
        for (int n = N - 1; n >= 0; n--)
            if (above[n]) for (int a = 0; a < g.nodes[n].nargs; a++) above[g.nodes[n].args[a]] = 1;

        Builder b(g);
        std::vector<int> adj(N, -1);                        // accumulated cotangent of each node
        // `pattern` is the broadcast pattern of the value the contribution comes through (the forward
        // consumer of n): the contribution stands for one term per index of that value, whether or not
        // its own expression varies there.  Along an axis where n is constant and the consumer is not,
        // n was used once per index, so the terms are summed: a contribution whose expression varies
        // there directly, one that is constant there (the cotangent of a sum handed on to an operand that
        // is itself constant along the summed axis) after it has been given one copy per index, so that
        // it counts extent times.  A cotangent wider than its value is summed the same way.
        auto accumulate_through = [&](int n, int contribution, uint32_t pattern) {
            if (!below[n] || !above[n] || b.failed) return;
            const uint32_t cb = g.nodes[contribution].bcast;
            const uint32_t over = g.nodes[n].bcast & ~(pattern & cb);
            if (over & cb) contribution = b.expand(contribution, over & cb);
            if (over) contribution = b.sum_over(contribution, over);
            adj[n] = adj[n] < 0 ? contribution : b.ap(EWF_ADD, adj[n], contribution);
        };
        for (int k = 0; k < ny; k++) accumulate_through(y[k], ybar[k], g.nodes[y[k]].bcast);

        for (int n = N - 1; n >= 0 && !b.failed; n--) {
            if (adj[n] < 0) continue;
            const Node nd = g.nodes[n];                     // copy: the vector grows below
            const int G = adj[n];
            const int a0 = nd.args[0], a1 = nd.args[1], a2 = nd.args[2];
            auto live = [&](int a) { return a >= 0 && below[a] && g.nodes[a].vtype == EWF_F32; };
            // a reduction hands its cotangent to an argument of its own pattern (every reduced element
            // receives it once); everything else is used once per index of the node's own pattern
            const uint32_t pattern = nd.kind == NodeKind::Reduce ? g.nodes[a0].bcast : nd.bcast;
            auto accumulate = [&](int a, int contribution) { accumulate_through(a, contribution, pattern); };
            switch (nd.kind) {
            case NodeKind::Cast:
                // float32 and float16 casts pass the cotangent through (rounding has derivative one
                // almost everywhere); a cast to or from int32 stops it
                if (nd.op != EWF_I32 && live(a0)) accumulate(a0, G);
                break;
            case NodeKind::Reduce:
                if (!live(a0)) break;
                if (nd.op == EWF_RSUM) accumulate(a0, G);
                else if (nd.op == EWF_RMAX || nd.op == EWF_RMIN)    // every element equal to the extreme value receives it
                    accumulate(a0, b.ap(EWF_WHERE, b.ap(EWF_EQ, a0, n), G, b.lit(0.0)));
                else if (nd.op == EWF_RPROD) {
                    // d(prod)/dx_i is the product of the other elements.  With no zero among the reduced
                    // elements that is prod / x_i; with exactly one zero only that element has a non-zero
                    // derivative (the product of the non-zero ones); with more, every derivative is zero.
                    const int z = b.lit(0.0), one = b.lit(1.0);
                    const int is_zero = b.ap(EWF_EQ, a0, z);
                    Node r; r.kind = NodeKind::Reduce; r.nargs = 1; r.axes = nd.axes; r.keep = true;
                    r.op = EWF_RSUM; r.args[0] = b.ap(EWF_WHERE, is_zero, one, z);
                    const int zeros = b.push(r);
                    r.op = EWF_RPROD; r.args[0] = b.ap(EWF_WHERE, is_zero, one, a0);
                    const int others = b.push(r);
                    const int at_zero = b.ap(EWF_WHERE, b.ap(EWF_EQ, zeros, one), others, z);
                    const int elsewhere = b.ap(EWF_WHERE, b.ap(EWF_EQ, zeros, z), b.ap(EWF_DIV, others, a0), z);
                    accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_WHERE, is_zero, at_zero, elsewhere)));
                }
                break;
            case NodeKind::Apply:
                switch (nd.op) {
                case EWF_ADD: if (live(a0)) accumulate(a0, G); if (live(a1)) accumulate(a1, G); break;
                case EWF_SUB: if (live(a0)) accumulate(a0, G); if (live(a1)) accumulate(a1, b.ap(EWF_NEG, G)); break;
                case EWF_MUL: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, a1)); if (live(a1)) accumulate(a1, b.ap(EWF_MUL, G, a0)); break;
                case EWF_DIV:
                    if (live(a0)) accumulate(a0, b.ap(EWF_DIV, G, a1));
                    if (live(a1)) accumulate(a1, b.ap(EWF_NEG, b.ap(EWF_DIV, b.ap(EWF_MUL, G, n), a1)));
                    break;
                case EWF_NEG: if (live(a0)) accumulate(a0, b.ap(EWF_NEG, G)); break;
                case EWF_ABS:
                    if (live(a0)) {
                        int z = b.lit(0.0);
                        accumulate(a0, b.ap(EWF_WHERE, b.ap(EWF_GT, a0, z), G, b.ap(EWF_WHERE, b.ap(EWF_LT, a0, z), b.ap(EWF_NEG, G), z)));
                    }
                    break;
                case EWF_EXP: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, n)); break;
                case EWF_EXPM1: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_ADD, n, b.lit(1.0)))); break;
                case EWF_LOG: if (live(a0)) accumulate(a0, b.ap(EWF_DIV, G, a0)); break;
                case EWF_LOG1P: if (live(a0)) accumulate(a0, b.ap(EWF_DIV, G, b.ap(EWF_ADD, a0, b.lit(1.0)))); break;
                case EWF_SQRT: if (live(a0)) accumulate(a0, b.ap(EWF_DIV, G, b.ap(EWF_MUL, b.lit(2.0), n))); break;
                case EWF_SQR: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_MUL, b.lit(2.0), a0))); break;
                case EWF_RECIP: if (live(a0)) accumulate(a0, b.ap(EWF_NEG, b.ap(EWF_MUL, G, b.ap(EWF_SQR, n)))); break;
                case EWF_TANH: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_SUB, b.lit(1.0), b.ap(EWF_SQR, n)))); break;
                case EWF_SIGMOID: if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_MUL, n, b.ap(EWF_SUB, b.lit(1.0), n)))); break;
                case EWF_MAX: case EWF_MIN: {
                    // the first operand takes the cotangent where it is the result (ties included)
                    int first = b.ap(nd.op == EWF_MAX ? EWF_GE : EWF_LE, a0, a1);
                    int z = b.lit(0.0);
                    if (live(a0)) accumulate(a0, b.ap(EWF_WHERE, first, G, z));
                    if (live(a1)) accumulate(a1, b.ap(EWF_WHERE, first, z, G));
                    break;
                }
                case EWF_POW:
                    if (live(a0)) accumulate(a0, b.ap(EWF_MUL, G, b.ap(EWF_MUL, a1, b.ap(EWF_POW, a0, b.ap(EWF_SUB, a1, b.lit(1.0))))));
                    if (live(a1)) accumulate(a1, b.ap(EWF_MUL, G, b.ap(EWF_MUL, n, b.ap(EWF_LOG, a0))));
                    break;
                case EWF_WHERE: {
                    int z = b.lit(0.0);
                    if (live(a1)) accumulate(a1, b.ap(EWF_WHERE, a0, G, z));
                    if (live(a2)) accumulate(a2, b.ap(EWF_WHERE, a0, z, G));
                    break;
                }
                default: break;                             // comparisons: piecewise constant
                }
                break;
            default: break;                                 // inputs, scalars, literals, iota: leaves
            }
        }
        if (b.failed) return EWF_EINVAL;
        for (int j = 0; j < nwrt; j++) {
            int v = adj[wrt[j]];
            if (v < 0) {
                // no differentiated value depends on it: a zero with the value's own pattern
                v = b.ap(EWF_MUL, wrt[j], b.lit(0.0));
            }
            // an accumulated cotangent may be constant where the value varies (the gradient of a plain
            // sum is the same for every element): the result takes the value's own pattern
            const uint32_t narrow = g.nodes[v].bcast & ~g.nodes[wrt[j]].bcast;
            if (narrow) v = b.expand(v, narrow);
            if (b.failed) return EWF_EINVAL;
            grads[j] = v;
        }
        return EWF_OK;
    });
}
