// The generator's common part: the state of one generation (struct Gen), the emitters every
// kernel class shares (values of the scalar graph, accumulator structs, the second kernel that
// folds partial results) and small text helpers.  One source file per kernel class implements
// Gen::gen_tile, Gen::gen_row and Gen::gen_col.
#ifndef EWF_GEN_H
#define EWF_GEN_H

#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <sstream>

#include "ewf_internal.h"

namespace ewf {

inline const char *ctype(ewf_dtype t) { return t == EWF_F16 ? "ewf_half" : t == EWF_I32 ? "int" : "float"; }
inline const char *vtype_c(ewf_dtype t) { return t == EWF_I32 ? "int" : "float"; }
inline int isz(ewf_dtype t) { return t == EWF_F16 ? 2 : 4; }

inline std::string f32_literal(double v)
{
    float f = (float)v;
    uint32_t b;
    memcpy(&b, &f, 4);
    char buf[64];
    snprintf(buf, sizeof buf, "ewf_bits_f32(0x%08xu)", b);
    return buf;
}

inline std::string i32_literal(double v)
{
    int64_t w = (int64_t)v;
    uint32_t b = (uint32_t)(uint64_t)w;
    char buf[64];
    snprintf(buf, sizeof buf, "((int)0x%08xu)", b);
    return buf;
}

// assigns offsets and the total size with C layout rules (ewf_codegen.cpp)
void finish_layout(ParamLayout &L);

struct EmitCtx {
    std::function<std::string(int)> input;     // expression of input k (already a value type)
    std::function<std::string(int)> coord;     // expression of the coordinate on canonical dim d
};

struct Gen {
    const Exec &e;
    Plan &p;
    const Graph &g;
    const Canon &c;
    const ReduceInfo &red;
    std::ostringstream o;
    int R;
    int VEC;
    std::vector<char> is_level, is_cross;     // per node
    std::vector<char> after_cross;
    std::vector<char> live;
    std::vector<char> nonneg, positive;       // sign facts provable from the graph alone
    // Values that reach the outputs only as terms of a float32 sum.  The bar for such outputs
    // is the reduction bar (1e-5 relative), which the native-rate routines with fix-ups meet in
    // the worst case (exp: at most 6e-8 * (1 + |x| log2 e) relative, under 6e-6 wherever the
    // result is finite), so under the automatic math mode these nodes use that flavour.
    std::vector<char> sum_only;
    // Values that feed a product, an extreme value or an arg-max (see the constructor): these keep
    // the accurate routines throughout.
    std::vector<char> strict;

    // A small sign analysis over the scalar graph, in the spirit of the specialisation stage
    // of paper section 2.2.1: when the base of a power is provably positive (x*x + 1, exp(u),
    // a positive literal ...) the cheap exp2(y*log2(x)) form needs no sign handling.
    void analyse_signs()
    {
        const int N = (int)g.nodes.size();
        nonneg.assign(N, 0); positive.assign(N, 0);
        for (int n = 0; n < N; n++) {
            const Node &nd = g.nodes[n];
            if (nd.vtype != EWF_F32) continue;
            auto P = [&](int a) { return positive[nd.args[a]] != 0; };
            auto Z = [&](int a) { return nonneg[nd.args[a]] != 0; };
            bool pos = false, nn = false;
            switch (nd.kind) {
            case NodeKind::Const: pos = nd.cval > 0 && (float)nd.cval > 0.0f; nn = nd.cval >= 0; break;
            case NodeKind::Cast: if (g.nodes[nd.args[0]].vtype == EWF_F32 && nd.op != EWF_I32) { nn = Z(0); pos = nd.op == EWF_F32 && P(0); } break;
            case NodeKind::Reduce:
                if (nd.op == EWF_RSUM || nd.op == EWF_RMAX || nd.op == EWF_RMIN) nn = Z(0);
                if (nd.op == EWF_RMAX || nd.op == EWF_RMIN) pos = P(0);
                break;
            case NodeKind::Apply:
                switch (nd.op) {
                case EWF_ABS: case EWF_SQR: case EWF_SQRT: nn = true; break;
                case EWF_EXP: nn = true; break;            // may underflow to zero
                case EWF_SIGMOID: nn = true; break;
                case EWF_MUL: nn = (nd.args[0] == nd.args[1]) || (Z(0) && Z(1)); break;
                case EWF_ADD: nn = Z(0) && Z(1); pos = nn && (P(0) || P(1)); break;
                case EWF_DIV: nn = Z(0) && P(1); break;
                case EWF_RECIP: nn = P(0); break;
                case EWF_MAX: nn = Z(0) || Z(1); pos = P(0) || P(1); break;
                case EWF_MIN: nn = Z(0) && Z(1); pos = P(0) && P(1); break;
                case EWF_WHERE: nn = Z(1) && Z(2); pos = P(1) && P(2); break;
                case EWF_LOG1P: nn = Z(0); break;
                case EWF_EXPM1: nn = Z(0); break;
                case EWF_TANH: nn = Z(0); break;
                default: break;
                }
                break;
            default: break;
            }
            positive[n] = pos; nonneg[n] = nn || pos;
        }
    }

    Gen(const Exec &e_, Plan &p_) : e(e_), p(p_), g(e_.g), c(p_.canon), red(p_.red)
    {
        R = c.rank;
        VEC = c.vec;
        const int N = (int)g.nodes.size();
        is_level.assign(N, 0); is_cross.assign(N, 0); after_cross.assign(N, 0); live.assign(N, 0);
        for (int n : red.level_nodes) is_level[n] = 1;
        for (int n : red.cross_nodes) is_cross[n] = 1;
        for (const OutputDecl &od : g.outputs) live[od.value] = 1;
        for (int n = N - 1; n >= 0; n--)
            if (live[n]) for (int a = 0; a < g.nodes[n].nargs; a++) live[g.nodes[n].args[a]] = 1;
        for (int n = 0; n < N; n++) {
            if (is_cross[n]) after_cross[n] = 1;
            for (int a = 0; a < g.nodes[n].nargs; a++) if (after_cross[g.nodes[n].args[a]]) after_cross[n] = 1;
        }
        analyse_signs();
        // Which values must meet the element-wise bar: those that reach an output that depends on
        // no reduction, through no float32 sum.  An output computed from a reduction is held to the
        // bar for reductions (1e-5), which the native-rate flavour with fix-ups meets (see sum_only).
        std::vector<char> direct(N, 0), below_reduce(N, 0);
        for (int n = 0; n < N; n++) {
            const Node &nd = g.nodes[n];
            if (nd.kind == NodeKind::Reduce && real_reduce(n)) below_reduce[n] = 1;
            for (int a = 0; a < nd.nargs; a++) if (below_reduce[nd.args[a]]) below_reduce[n] = 1;
        }
        for (const OutputDecl &od : g.outputs) if (!below_reduce[od.value]) direct[od.value] = 1;
        // (what a product, maximum, minimum or arg-max folds stays accurate: a product compounds
        // the error of its factors, and an extreme value or its index can flip on a rounding)
        strict.assign(N, 0);
        for (int n = 0; n < N; n++) {
            const Node &nd = g.nodes[n];
            if (live[n] && nd.kind == NodeKind::Reduce && real_reduce(n) && !(nd.op == EWF_RSUM && nd.vtype == EWF_F32) &&
                nd.op != kRSumExpShifted) direct[nd.args[0]] = strict[nd.args[0]] = 1;
        }
        // (likewise what a comparison or a conversion to an integer reads: the outcome is discrete.
        // A plan in several kernels evaluates such a value in more than one of them -- the
        // elements equal to a maximum that an earlier kernel folded -- and they must agree to the
        // last bit, so all of them take the accurate routines.)
        for (int n = 0; n < N; n++) {
            const Node &nd = g.nodes[n];
            if (!live[n] || nd.vtype != EWF_I32) continue;
            const bool cmp = nd.kind == NodeKind::Apply && (nd.op == EWF_GT || nd.op == EWF_GE || nd.op == EWF_LT || nd.op == EWF_LE ||
                                                            nd.op == EWF_EQ || nd.op == EWF_NE);
            const bool to_int = nd.kind == NodeKind::Cast && nd.op == EWF_I32;
            if (!cmp && !to_int) continue;
            for (int a = 0; a < nd.nargs; a++)
                if (g.nodes[nd.args[a]].vtype == EWF_F32) direct[nd.args[a]] = strict[nd.args[a]] = 1;
        }
        for (int n = N - 1; n >= 0; n--) {
            if (!direct[n]) continue;
            const Node &nd = g.nodes[n];
            if (nd.kind == NodeKind::Reduce && nd.op == EWF_RSUM && nd.vtype == EWF_F32 && real_reduce(n)) continue;
            for (int a = 0; a < nd.nargs; a++) { direct[nd.args[a]] = 1; if (strict[n]) strict[nd.args[a]] = 1; }
        }
        sum_only.assign(N, 0);
        for (int n = 0; n < N; n++) sum_only[n] = live[n] && !direct[n];
    }

    bool real_reduce(int n) const { return is_level[n] || is_cross[n]; }

    std::string opname(int k) const
    {
        const Operand &op = c.ops[k];
        return (op.is_output ? "out" : "in") + std::to_string(op.index);
    }

    // Marks the ancestors of `targets`, stopping at materialised reductions.
    std::vector<char> needed(const std::vector<int> &targets) const
    {
        const int N = (int)g.nodes.size();
        std::vector<char> need(N, 0);
        for (int t : targets) need[t] = 1;
        for (int n = N - 1; n >= 0; n--) {
            if (!need[n]) continue;
            const Node &nd = g.nodes[n];
            if (nd.kind == NodeKind::Reduce && real_reduce(n)) {
                continue;                       // read from its result variable
            }
            for (int a = 0; a < nd.nargs; a++) need[nd.args[a]] = 1;
        }
        return need;
    }

    std::vector<int> inputs_of(const std::vector<char> &need) const
    {
        std::vector<int> ks;
        for (size_t n = 0; n < need.size(); n++)
            if (need[n] && g.nodes[n].kind == NodeKind::Input) ks.push_back(g.nodes[n].index);
        return ks;
    }

    // Emits `const T v<n> = ...;` for every needed node, in graph order.
    void emit_values(const std::vector<char> &need, const EmitCtx &cx, const std::string &ind)
    {
        for (size_t n = 0; n < need.size(); n++) {
            if (!need[n]) continue;
            const Node &nd = g.nodes[n];
            // Under the automatic math mode the sigmoid and the hyperbolic tangent of a float32
            // result take the native-rate routines too: both are bounded, their relative error
            // stays under 1.5e-6 (the exponential's argument is never large where its value
            // matters) and their absolute error under 1.2e-7, inside the element-wise bar.
            const bool bounded = nd.kind == NodeKind::Apply && (nd.op == EWF_TANH || nd.op == EWF_SIGMOID) && !strict[n];
            const int fl = (e.auto_math && e.math_flavour == 1 && (sum_only[n] || bounded)) ? 2 : e.math_flavour;
            const char *M = fl == 3 ? "ewf_bare" : fl == 2 ? "ewf_fast" : "ewf_acc";
            std::string a0 = nd.nargs > 0 ? "v" + std::to_string(nd.args[0]) : "";
            std::string a1 = nd.nargs > 1 ? "v" + std::to_string(nd.args[1]) : "";
            std::string a2 = nd.nargs > 2 ? "v" + std::to_string(nd.args[2]) : "";
            const bool isint = nd.nargs > 0 && g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string rhs;
            switch (nd.kind) {
            case NodeKind::Input: rhs = cx.input(nd.index); break;
            case NodeKind::Scalar: rhs = "p.s" + std::to_string(nd.index); break;
            case NodeKind::Const: rhs = nd.vtype == EWF_I32 ? i32_literal(nd.cval) : f32_literal(nd.cval); break;
            case NodeKind::Iota: {
                int cd = c.orig_of_axis[nd.index];
                rhs = cd < 0 ? "0" : "(int)(" + cx.coord(cd) + ")";
                break;
            }
            case NodeKind::Cast:
                if (nd.op == EWF_F16) rhs = "ewf_round_f16(" + a0 + ")";
                else if (nd.op == EWF_F32) rhs = isint ? "(float)" + a0 : a0;
                else rhs = isint ? a0 : "ewf_f2i(" + a0 + ")";
                break;
            case NodeKind::Reduce:
                if (real_reduce((int)n)) rhs = "r" + std::to_string(n);
                else if (nd.op == kRSumExpShifted) rhs = std::string(M) + "::exp(" + a0 + " - " + a0 + ")";   // one term: exp(x - x)
                else if (nd.op == kRSumSqCentred) rhs = "(" + a0 + " - " + a0 + ") * (" + a0 + " - " + a0 + ")";   // one term: (x - x)^2
                else rhs = (nd.op == EWF_RARGMAX) ? "0" : a0;      // reduction over extent-1 axes
                break;
            case NodeKind::Apply:
                switch (nd.op) {
                case EWF_ADD: rhs = isint ? "ewf_addi(" + a0 + ", " + a1 + ")" : a0 + " + " + a1; break;
                case EWF_SUB: rhs = isint ? "ewf_subi(" + a0 + ", " + a1 + ")" : a0 + " - " + a1; break;
                case EWF_MUL: rhs = isint ? "ewf_muli(" + a0 + ", " + a1 + ")" : a0 + " * " + a1; break;
                case EWF_SQR: rhs = isint ? "ewf_muli(" + a0 + ", " + a0 + ")" : a0 + " * " + a0; break;
                case EWF_DIV: rhs = std::string(M) + "::div(" + a0 + ", " + a1 + ")"; break;
                case EWF_NEG: rhs = isint ? "ewf_negi(" + a0 + ")" : "-" + a0; break;
                case EWF_ABS: rhs = "ewf_abs(" + a0 + ")"; break;
                case EWF_EXP: {
                    // exp(k * s), k a literal, with the native-rate flavours: one multiplication
                    // by k * log2 e (folded here) and the hardware exp2
                    const Node &arg = g.nodes[nd.args[0]];
                    int kside = -1;
                    if (fl >= 2 && arg.kind == NodeKind::Apply && arg.op == EWF_MUL)
                        for (int sd = 0; sd < 2; sd++) if (g.nodes[arg.args[sd]].kind == NodeKind::Const) kside = sd;
                    if (kside >= 0) {
                        const double k = (double)(float)g.nodes[arg.args[kside]].cval;
                        rhs = "__builtin_amdgcn_exp2f(v" + std::to_string(arg.args[1 - kside]) + " * " + f32_literal(k * 1.44269504088896340736) + ")";
                    } else {
                        rhs = std::string(M) + "::exp(" + a0 + ")";
                    }
                    break;
                }
                case EWF_LOG: rhs = std::string(M) + "::log(" + a0 + ")"; break;
                case EWF_LOG1P: rhs = std::string(M) + "::log1p(" + a0 + ")"; break;
                case EWF_EXPM1: rhs = std::string(M) + "::expm1(" + a0 + ")"; break;
                case EWF_SQRT: rhs = std::string(M) + "::sqrt(" + a0 + ")"; break;
                case EWF_TANH: rhs = std::string(M) + "::tanh(" + a0 + ")"; break;
                case EWF_SIGMOID: rhs = std::string(M) + "::sigmoid(" + a0 + ")"; break;
                case EWF_RECIP: rhs = std::string(M) + "::recip(" + a0 + ")"; break;
                case EWF_POW: rhs = std::string(M) + (positive[nd.args[0]] ? "::pow_pos(" : "::pow(") + a0 + ", " + a1 + ")"; break;
                case EWF_MAX: rhs = "ewf_max(" + a0 + ", " + a1 + ")"; break;
                case EWF_MIN: rhs = "ewf_min(" + a0 + ", " + a1 + ")"; break;
                case EWF_WHERE: rhs = "(ewf_truth(" + a0 + ") ? " + a1 + " : " + a2 + ")"; break;
                case EWF_GT: rhs = "(int)(" + a0 + " > " + a1 + ")"; break;
                case EWF_GE: rhs = "(int)(" + a0 + " >= " + a1 + ")"; break;
                case EWF_LT: rhs = "(int)(" + a0 + " < " + a1 + ")"; break;
                case EWF_LE: rhs = "(int)(" + a0 + " <= " + a1 + ")"; break;
                case EWF_EQ: rhs = "(int)(" + a0 + " == " + a1 + ")"; break;
                case EWF_NE: rhs = "(int)(" + a0 + " != " + a1 + ")"; break;
                default: rhs = "0"; break;
                }
                break;
            }
            o << ind << "const " << vtype_c(nd.vtype) << " v" << n << " = " << rhs << ";\n";
        }
    }

    // ---- accumulators -------------------------------------------------------------------

    // A maximum over the same argument as an arg-max of the same list needs no slot of its
    // own: the arg-max already carries the running maximum (with the same NaN rule).
    // Returns the arg-max's slot, or -1.
    int shared_slot(const std::vector<int> &nodes, size_t i) const
    {
        const Node &nd = g.nodes[nodes[i]];
        if (nd.op != EWF_RMAX) return -1;
        for (size_t j = 0; j < nodes.size(); j++) {
            const Node &o2 = g.nodes[nodes[j]];
            if (o2.op == EWF_RARGMAX && o2.args[0] == nd.args[0] && o2.axes == nd.axes) return (int)j;
        }
        return -1;
    }

    size_t acc_bytes(const std::vector<int> &nodes) const
    {
        size_t b = 0;
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            const int op = g.nodes[nodes[i]].op;
            b += op == kRSumSqCentred ? 12 : (op == EWF_RARGMAX || op == kRSumExpShifted) ? 8 : 4;
        }
        return b;
    }

    // the exponential inside a sum: under the automatic math mode the native-rate flavour with
    // fix-ups (see sum_only)
    const char *sum_math() const
    {
        const int fl = (e.auto_math && e.math_flavour == 1) ? 2 : e.math_flavour;
        return fl == 3 ? "ewf_bare" : fl == 2 ? "ewf_fast" : "ewf_acc";
    }

    // Declares `struct <name>` with one slot per reduction in `nodes`, its identity and its
    // combine function.
    void emit_acc_struct(const std::string &name, const std::vector<int> &nodes)
    {
        o << "struct " << name << " {\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            const Node &nd = g.nodes[nodes[i]];
            const Node &arg = g.nodes[nd.args[0]];
            if (nd.op == EWF_RARGMAX) o << "    " << vtype_c(arg.vtype) << " a" << i << "; int i" << i << ";\n";
            else if (nd.op == kRSumExpShifted) o << "    float a" << i << ", b" << i << ";      // running maximum, sum of exp(x - maximum)\n";
            else if (nd.op == kRSumSqCentred) o << "    float n" << i << ", a" << i << ", b" << i << ";      // count, running mean, sum of squared deviations from it\n";
            else o << "    " << vtype_c(nd.vtype) << " a" << i << ";\n";
        }
        o << "};\n";
        o << "EWF_DEV " << name << " " << name << "_identity()\n{\n    " << name << " a;\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string id;
            switch (nd.op) {
            case EWF_RSUM: id = isint ? "0" : "0.0f"; break;
            case EWF_RPROD: id = isint ? "1" : "1.0f"; break;
            case EWF_RMAX: case EWF_RARGMAX: id = isint ? "(-2147483647 - 1)" : "ewf_bits_f32(0xff800000u)"; break;
            case EWF_RMIN: id = isint ? "2147483647" : "ewf_bits_f32(0x7f800000u)"; break;
            // the most negative finite number, not -inf: x - maximum then never is inf - inf
            // for an element that is -inf, and exp(x - maximum) is 0 for it as it should be
            case kRSumExpShifted: id = "ewf_bits_f32(0xff7fffffu)"; o << "    a.b" << i << " = 0.0f;\n"; break;
            case kRSumSqCentred: id = "0.0f"; o << "    a.n" << i << " = 0.0f;\n    a.b" << i << " = 0.0f;\n"; break;
            }
            o << "    a.a" << i << " = " << id << ";\n";
            if (nd.op == EWF_RARGMAX) o << "    a.i" << i << " = 2147483647;\n";
        }
        o << "    return a;\n}\n";
        o << "struct " << name << "_combine {\n    EWF_DEV " << name << " operator()(const " << name << " &x, const "
          << name << " &y) const\n    {\n        " << name << " r;\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string a = "x.a" + std::to_string(i), b = "y.a" + std::to_string(i);
            switch (nd.op) {
            case EWF_RSUM: o << "        r.a" << i << " = " << (isint ? "ewf_addi(" + a + ", " + b + ")" : a + " + " + b) << ";\n"; break;
            case EWF_RPROD: o << "        r.a" << i << " = " << (isint ? "ewf_muli(" + a + ", " + b + ")" : a + " * " + b) << ";\n"; break;
            case EWF_RMAX: o << "        r.a" << i << " = ewf_max(" << a << ", " << b << ");\n"; break;
            case EWF_RMIN: o << "        r.a" << i << " = ewf_min(" << a << ", " << b << ");\n"; break;
            case kRSumExpShifted:
                // both sums are rescaled to the common maximum
                o << "        r.a" << i << " = ewf_max(" << a << ", " << b << ");\n"
                  << "        r.b" << i << " = x.b" << i << " * " << sum_math() << "::exp(" << a << " - r.a" << i << ") + y.b" << i << " * "
                  << sum_math() << "::exp(" << b << " - r.a" << i << ");\n";
                break;
            case kRSumSqCentred:
                // two groups of elements become one: the means meet at their weighted average and
                // the distance between them adds to the squared deviations
                o << "        { const float n_ = x.n" << i << " + y.n" << i << ";\n"
                  << "          const float r_ = n_ > 0.0f ? 1.0f / n_ : 0.0f;\n"
                  << "          const float d_ = " << b << " - " << a << ";\n"
                  << "          r.n" << i << " = n_;\n"
                  << "          r.a" << i << " = " << a << " + d_ * (y.n" << i << " * r_);\n"
                  << "          r.b" << i << " = x.b" << i << " + y.b" << i << " + d_ * d_ * (x.n" << i << " * y.n" << i << " * r_); }\n";
                break;
            case EWF_RARGMAX: {
                std::string ia = "x.i" + std::to_string(i), ib = "y.i" + std::to_string(i);
                if (isint) {
                    o << "        { const bool t = (" << b << " > " << a << ") | ((" << b << " == " << a << ") & (" << ib << " < " << ia << "));\n";
                } else {
                    // NaN ranks above every number; equal keys keep the lower index.  (Plain
                    // and / or of the comparison results, not the short-circuit forms: those
                    // become branches in every step of a lane fold.)
                    o << "        { const bool gt = (" << b << " > " << a << ") | ((" << b << " != " << b << ") & (" << a << " == " << a << "));\n"
                      << "          const bool eq = (" << b << " == " << a << ") | ((" << b << " != " << b << ") & (" << a << " != " << a << "));\n"
                      << "          const bool t = gt | (eq & (" << ib << " < " << ia << "));\n";
                }
                o << "          r.a" << i << " = t ? " << b << " : " << a << "; r.i" << i << " = t ? " << ib << " : " << ia << "; }\n";
                break;
            }
            }
        }
        o << "        return r;\n    }\n};\n";
    }

    // Assigns r<n> for each reduction from the folded accumulator.
    void emit_results(const std::string &acc, const std::vector<int> &nodes, const std::string &ind)
    {
        for (size_t i = 0; i < nodes.size(); i++) {
            const Node &nd = g.nodes[nodes[i]];
            const int sh = shared_slot(nodes, i);
            if (nd.op == EWF_RARGMAX) o << ind << "const int r" << nodes[i] << " = " << acc << ".i" << i << ";\n";
            else if (nd.op == kRSumExpShifted)
                // no term at all (every element -inf) or a maximum of +inf: x - max(x) is
                // inf - inf for some element, so the sum as described is NaN
                o << ind << "const float r" << nodes[i] << " = (" << acc << ".b" << i << " == 0.0f || " << acc << ".a" << i
                  << " == ewf_bits_f32(0x7f800000u)) ? ewf_bits_f32(0x7fc00000u) : " << acc << ".b" << i << ";\n";
            else if (nd.op == kRSumSqCentred) o << ind << "const float r" << nodes[i] << " = " << acc << ".b" << i << ";\n";
            else o << ind << "const " << vtype_c(nd.vtype) << " r" << nodes[i] << " = " << acc << ".a" << (sh >= 0 ? sh : (int)i) << ";\n";
        }
    }

    // Folds one element into every slot of the accumulator `acc` (slot-wise, no temporaries).
    // With `ascending` the caller guarantees that one thread meets the indices of an arg-max
    // in increasing order: a later element then replaces the running maximum only when it is
    // strictly greater (or the first NaN), and the index comparison falls away.  The
    // identity index (no element taken yet) must then be resolved by emit_first_index.
    // `only` (one flag per position of `nodes`, or null for all) restricts it to some slots.
    void emit_accumulate(const std::string &acc, const std::vector<int> &nodes,
                         const std::function<std::string(int)> &argmax_index, const std::string &ind,
                         bool ascending = false, const std::vector<char> *only = nullptr)
    {
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            if (only && !(*only)[i]) continue;
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string a = acc + ".a" + std::to_string(i), v = "v" + std::to_string(nd.args[0]);
            switch (nd.op) {
            case EWF_RSUM: o << ind << a << " = " << (isint ? "ewf_addi(" + a + ", " + v + ")" : a + " + " + v) << ";\n"; break;
            case EWF_RPROD: o << ind << a << " = " << (isint ? "ewf_muli(" + a + ", " + v + ")" : a + " * " + v) << ";\n"; break;
            case EWF_RMAX: o << ind << a << " = ewf_max(" << a << ", " << v << ");\n"; break;
            case EWF_RMIN: o << ind << a << " = ewf_min(" << a << ", " << v << ");\n"; break;
            case kRSumExpShifted: {
                // exp(-|x - maximum|) serves both cases: it rescales the sum when x is the new
                // maximum and is the new term otherwise
                const std::string b = acc + ".b" + std::to_string(i);
                o << ind << "{ const float d_ = " << v << " - " << a << ";\n"
                  << ind << "  const float w_ = " << sum_math() << "::exp(-__builtin_fabsf(d_));\n"
                  << ind << "  " << b << " = d_ > 0.0f ? " << b << " * w_ + 1.0f : " << b << " + w_;\n"
                  << ind << "  " << a << " = ewf_max(" << a << ", " << v << "); }\n";
                break;
            }
            case kRSumSqCentred: {
                // the single-pass update: the mean moves by its share of the new deviation, and
                // the product of the deviations before and after the move is the element's part
                const std::string nn = acc + ".n" + std::to_string(i), b = acc + ".b" + std::to_string(i);
                o << ind << "{ " << nn << " += 1.0f;\n"
                  << ind << "  const float d_ = " << v << " - " << a << ";\n"
                  << ind << "  " << a << " = __builtin_fmaf(d_, __builtin_amdgcn_rcpf(" << nn << "), " << a << ");\n"
                  << ind << "  " << b << " = __builtin_fmaf(d_, " << v << " - " << a << ", " << b << "); }\n";
                break;
            }
            case EWF_RARGMAX: {
                std::string ia = acc + ".i" + std::to_string(i);
                std::string ib = "(int)(" + argmax_index(nodes[i]) + ")";
                if (ascending && isint) {
                    o << ind << "{ const bool t = " << v << " > " << a << ";\n";
                } else if (ascending) {
                    // greater, or the first NaN; a NaN already held stays
                    o << ind << "{ const bool t = !(" << v << " <= " << a << ") & (" << a << " == " << a << ");\n";
                } else if (isint) {
                    o << ind << "{ const bool t = (" << v << " > " << a << ") | ((" << v << " == " << a << ") & (" << ib << " < " << ia << "));\n";
                } else {
                    o << ind << "{ const bool gt = (" << v << " > " << a << ") | ((" << v << " != " << v << ") & (" << a << " == " << a << "));\n"
                      << ind << "  const bool eq = (" << v << " == " << a << ") | ((" << v << " != " << v << ") & (" << a << " != " << a << "));\n"
                      << ind << "  const bool t = gt | (eq & (" << ib << " < " << ia << "));\n";
                }
                o << ind << "  " << a << " = t ? " << v << " : " << a << "; " << ia << " = t ? " << ib << " : " << ia << "; }\n";
                break;
            }
            }
        }
    }

    // Slots that can take a whole vector of elements at once (float32 arguments): the running
    // maximum of a sum of shifted exponentials, of a maximum and -- met in ascending order -- of an
    // arg-max.  Returns one flag per position of `nodes`.
    std::vector<char> vector_slots(const std::vector<int> &nodes, bool ascending) const
    {
        std::vector<char> f(nodes.size(), 0);
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
            const Node &nd = g.nodes[nodes[i]];
            if (g.nodes[nd.args[0]].vtype != EWF_F32) continue;
            f[i] = nd.op == kRSumExpShifted || nd.op == EWF_RMAX || (nd.op == EWF_RARGMAX && ascending);
        }
        return f;
    }

    // Folds the VEC values xs[0..VEC) of argument `arg` into the slots flagged in `slots` that
    // take this argument.  When all of them are finite (and no slot holds a NaN) a vector costs
    // one hardware maximum per element, and per slot: for a maximum or arg-max a comparison (the
    // index is looked up only when the maximum moves, which becomes rare quickly); for a sum of
    // shifted exponentials one rescaling of the sum and one exponential per element, all against
    // the same new maximum.  Anything else -- a NaN or an infinity among the values, a NaN held,
    // a vector cut short by the row's end (`full` false) -- goes element by element through
    // emit_accumulate, whose rules for those cases the fast path never has to reproduce.
    void emit_vector_accumulate(const std::string &acc, const std::vector<int> &nodes, const std::vector<char> &slots, int arg,
                                const std::string &xs, const std::string &full, const std::string &skip_element,
                                const std::function<std::string(int)> &argmax_index, const std::string &ind)
    {
        std::vector<char> mine(nodes.size(), 0);
        bool any = false;
        for (size_t i = 0; i < nodes.size(); i++) if (slots[i] && g.nodes[nodes[i]].args[0] == arg) { mine[i] = 1; any = true; }
        if (!any) return;
        o << ind << "{ float t_ = 0.0f;\n";
        o << ind << "  _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) t_ = __builtin_fmaf(" << xs << "[e_], 0.0f, t_);     // NaN iff a value is NaN or infinite\n";
        o << ind << "  bool fast_ = (t_ == 0.0f)";
        if (!full.empty()) o << " & (" << full << ")";
        for (size_t i = 0; i < nodes.size(); i++) if (mine[i]) o << " & (" << acc << ".a" << i << " == " << acc << ".a" << i << ")";
        o << ";\n";
        o << ind << "  if (fast_) {\n";
        o << ind << "      float vm_ = " << xs << "[0];\n";
        o << ind << "      _Pragma(\"unroll\") for (int e_ = 1; e_ < EWF_VEC; ++e_) vm_ = __builtin_fmaxf(vm_, " << xs << "[e_]);\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            if (!mine[i]) continue;
            const Node &nd = g.nodes[nodes[i]];
            const std::string a = acc + ".a" + std::to_string(i);
            if (nd.op == EWF_RMAX) {
                o << ind << "      " << a << " = __builtin_fmaxf(" << a << ", vm_);\n";
            } else if (nd.op == EWF_RARGMAX) {
                o << ind << "      if (vm_ > " << a << ") {\n";
                o << ind << "          int k_ = 0;\n";
                o << ind << "          _Pragma(\"unroll\") for (int e_ = EWF_VEC - 1; e_ >= 0; --e_) k_ = (" << xs << "[e_] == vm_) ? e_ : k_;\n";
                o << ind << "          const int e_ = k_;\n";
                o << ind << "          " << a << " = vm_; " << acc << ".i" << i << " = (int)(" << argmax_index(nodes[i]) << ");\n";
                o << ind << "      }\n";
            } else {
                const std::string b = acc + ".b" + std::to_string(i);
                o << ind << "      { const float mn_ = __builtin_fmaxf(" << a << ", vm_);\n";
                o << ind << "        float s_ = " << b << " * " << sum_math() << "::exp(" << a << " - mn_);\n";
                o << ind << "        _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) s_ += " << sum_math() << "::exp(" << xs << "[e_] - mn_);\n";
                o << ind << "        " << b << " = s_; " << a << " = mn_; }\n";
            }
        }
        o << ind << "  } else {\n";
        o << ind << "      _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        if (!skip_element.empty()) o << ind << "          if (" << skip_element << ") continue;\n";
        o << ind << "          const float v" << arg << " = " << xs << "[e_];\n";
        emit_accumulate(acc, nodes, argmax_index, ind + "          ", true, &mine);
        o << ind << "      }\n";
        o << ind << "  }\n";
        o << ind << "}\n";
    }

    // After an `ascending` accumulation: a thread whose elements all equal the identity value
    // (-inf, or the smallest integer) never replaced it, so its index is still the identity;
    // the first element it met is then the first occurrence of that maximum.
    void emit_first_index(const std::string &acc, const std::vector<int> &nodes, const std::string &has_first,
                          const std::string &first_index, const std::string &ind)
    {
        for (size_t i = 0; i < nodes.size(); i++)
            if (g.nodes[nodes[i]].op == EWF_RARGMAX)
                o << ind << "if (" << acc << ".i" << i << " == 2147483647 && (" << has_first << ")) " << acc << ".i" << i
                  << " = (int)(" << first_index << ");\n";
    }

    // "Sum over one axis of where(iota == T, X, 0)" with X a tensor input and T constant along
    // that axis has exactly one non-zero term: it is X read at index T (zero when T is out
    // of range).  The row class reads that element directly instead of comparing an index
    // per element.  Adding +0 keeps the sign rule of the sum (a sum of zeros is +0).
    struct Gather { int node, input, index_value, cdim; };
    bool match_gather(int n, Gather &out) const
    {
        const Node &nd = g.nodes[n];
        if (nd.kind != NodeKind::Reduce || nd.op != EWF_RSUM || nd.vtype != EWF_F32) return false;
        if (nd.axes & (nd.axes - 1)) return false;
        int axis = 0;
        while (!(nd.axes & (1u << axis))) axis++;
        const Node &w = g.nodes[nd.args[0]];
        if (w.kind != NodeKind::Apply || w.op != EWF_WHERE) return false;
        const Node &cnd = g.nodes[w.args[0]], &x = g.nodes[w.args[1]], &z = g.nodes[w.args[2]];
        if (z.kind != NodeKind::Const || z.cval != 0.0 || std::signbit(z.cval)) return false;
        if (x.kind != NodeKind::Input || (x.bcast & nd.axes)) return false;
        if (cnd.kind != NodeKind::Apply || cnd.op != EWF_EQ) return false;
        for (int side = 0; side < 2; side++) {
            const Node &io = g.nodes[cnd.args[side]], &t = g.nodes[cnd.args[1 - side]];
            if (io.kind == NodeKind::Iota && io.index == axis && t.vtype == EWF_I32 && (t.bcast & nd.axes)) {
                out = {n, x.index, cnd.args[1 - side], c.orig_of_axis[axis]};
                return out.cdim >= 0;
            }
        }
        return false;
    }

    // x / d for 0 <= x < n, d a literal that is not a power of two: the compiler's own
    // multiply-high runs at a quarter of the rate of the 24-bit multiply, and inside a tile every
    // index is small.  (x * m) >> s with m = ceil(2^s / d) is exact as long as x * (m * d - 2^s) <
    // 2^s; the smallest s for which that holds for all x < n with the product below 2^32 and both
    // factors below 2^24 is taken (none: the plain division).  The workgroups of the float16
    // stress workload's reading "B" spent an eighth of their vector cycles on such divisions.
    std::string div_small(const std::string &x, int64_t d, int64_t n) const
    {
        if (d <= 1) return x;
        if ((d & (d - 1)) == 0) { int sh = 0; while (((int64_t)1 << sh) < d) sh++; return "(" + x + " >> " + std::to_string(sh) + ")"; }
        if (n <= (int64_t)1 << 24)
            for (int sft = 1; sft < 32; sft++) {
                const int64_t m = (((int64_t)1 << sft) + d - 1) / d;
                if (m >= ((int64_t)1 << 24) || (n - 1) * m >= ((int64_t)1 << 32)) continue;
                if ((n - 1) * (m * d - ((int64_t)1 << sft)) < ((int64_t)1 << sft))
                    return "(int)(ewf_mul24(" + x + ", " + std::to_string(m) + ") >> " + std::to_string(sft) + ")";
            }
        return "(" + x + " / " + std::to_string(d) + ")";
    }
    // Statements that split `var` (below n) into `rem` = var % d and var /= d.
    std::string divmod_small(const std::string &rem, const std::string &var, int64_t d, int64_t n) const
    {
        if ((d & (d - 1)) == 0 || d >= ((int64_t)1 << 24))
            return rem + " = " + var + " % " + std::to_string(d) + "; " + var + " /= " + std::to_string(d) + ";";
        return "{ const int q_ = " + div_small(var, d, n) + "; " + rem + " = " + var + " - (int)ewf_mul24(q_, " + std::to_string(d) + "); " + var + " = q_; }";
    }

    // The canonical dimension of an arg-max axis; with several axes, of the first one that
    // has more than one element (-1 when there is none).
    int argmax_canon_dim(int node) const
    {
        const Node &nd = g.nodes[node];
        for (int d = 0; d < g.ndim; d++) if ((nd.axes & (1u << d)) && c.orig_of_axis[d] >= 0) return c.orig_of_axis[d];
        return -1;
    }
    // Number of arg-max axes with more than one element.
    int argmax_rank(int node) const
    {
        const Node &nd = g.nodes[node];
        int r = 0;
        for (int d = 0; d < g.ndim; d++) if ((nd.axes & (1u << d)) && c.orig_of_axis[d] >= 0) r++;
        return r;
    }
    // The index an arg-max returns for the element whose canonical coordinates `coord` names:
    // its position in the row-major order of the reduced axes, in axis order (one axis: the
    // coordinate itself).  An arg-max axis is never merged with a neighbour, so each has a
    // canonical dimension of its own whose extent is a kernel argument.
    std::string argmax_index(int node, const std::function<std::string(int)> &coord) const
    {
        const Node &nd = g.nodes[node];
        std::string s;
        for (int d = 0; d < g.ndim; d++) {
            if (!(nd.axes & (1u << d)) || c.orig_of_axis[d] < 0) continue;
            const std::string x = "(int)(" + coord(c.orig_of_axis[d]) + ")";
            s = s.empty() ? x : "(" + s + ") * (int)p.ext[" + std::to_string(c.orig_of_axis[d]) + "] + " + x;
        }
        return s.empty() ? std::string("0") : s;
    }

    // ---- common pieces ------------------------------------------------------------------

    void emit_header(int block)
    {
        o << "// generated by the fused element-wise + reduce library; do not edit\n";
        o << "#define EWF_BLOCK " << block << "\n";
        o << "#define EWF_NWAVES " << (block / 64) << "\n";
        o << "#define EWF_VEC " << VEC << "\n";
        o << "#define EWF_FIN_BLOCK 256\n";
        o << "typedef " << (c.idx64 ? "long long" : "int") << " idx_t;\n";
        // offsets inside a tile are never negative; when every operand spans less than 4 GiB
        // they are kept as 32-bit byte offsets from a uniform base
        o << "typedef " << (c.byte32 ? "unsigned" : "long long") << " ioff_t;\n";
    }

    void build_layout()
    {
        ParamLayout &L = p.layout;
        L.fields.clear();
        const ParamField::Type IDX = c.idx64 ? ParamField::I64 : ParamField::I32;
        for (size_t k = 0; k < c.ops.size(); k++) L.add(ParamField::Ptr, opname((int)k), 0);
        L.add(ParamField::Ptr, "ws_partials", 0);
        L.add(IDX, "ext", std::max(1, R));
        L.add(IDX, "ntile", std::max(1, R));
        L.add(IDX, "ntiles", 0);
        L.add(IDX, "nrows", 0);
        L.add(IDX, "nslots", 0);
        for (size_t k = 0; k < c.ops.size(); k++) L.add(IDX, "st_" + opname((int)k), std::max(1, R));
        for (int k = 0; k < g.nscalars; k++)
            L.add(g.nodes[g.scalar_node[k]].vtype == EWF_I32 ? ParamField::I32 : ParamField::F32, "s" + std::to_string(k), 0);
        finish_layout(L);
        o << L.declare("Params", c.idx64);
    }

    // typed base pointer of operand k at the (uniform) origin coordinates o<d>
    void emit_base(int k, const std::vector<int> &origin_dims, const std::string &ind)
    {
        const Operand &op = c.ops[k];
        std::string nm = opname(k), ty = ctype(op.storage);
        o << ind << (op.is_output ? "" : "const ") << ty << " *q_" << nm << " = (" << (op.is_output ? "" : "const ")
          << ty << " *)p." << nm;
        bool any = false;
        for (int d : origin_dims) {
            if (op.stride[d] == 0) continue;
            o << (any ? " + " : " + (") << "o" << d << " * p.st_" << nm << "[" << d << "]";
            any = true;
        }
        if (any) o << ")";
        o << ";\n";
    }

    int auto_waves_per_simd = 0;              // register budget the generator itself asks for

    std::string occupancy_attr() const
    {
        int w = (e.opts.waves_per_simd >= 1 && e.opts.waves_per_simd <= 8) ? e.opts.waves_per_simd : auto_waves_per_simd;
        if (w < 1) return "";
        return "__attribute__((amdgpu_waves_per_eu(" + std::to_string(w) + "))) ";
    }

    ewf_status fail(const std::string &why)
    {
        set_error("%s", why.c_str());
        return EWF_EUNSUPPORTED;
    }

    // Second kernel of the split reductions: one workgroup per reduction group; its lanes walk
    // the group's partials (contiguous in the workspace), a wavefront butterfly and an LDS
    // step in wavefront order fold them -- the same order on every run.
    // `inflight`: partials a thread loads before it folds them (more than one when a group has
    // many partials per thread, so that the loads overlap instead of each waiting for the last).
    // `gathers`: sums with a single non-zero term (see match_gather) that the streaming kernel
    // left out: the finishing thread reads that one element itself.
    void emit_finish_lanes(const std::vector<int> &level, const std::vector<int> &group_out_ops,
                           const std::string &nparts_expr, int fin_block, int inflight = 1,
                           const std::vector<Gather> &gathers = std::vector<Gather>())
    {
        o << "\n// folds the partials of each reduction group in a fixed order\n";
        o << "extern \"C\" __global__ void __launch_bounds__(" << fin_block << ") ewf_finish(const Params p)\n{\n";
        o << "    const int lane = threadIdx.x;\n";
        o << "    __shared__ Acc sm_fin[" << fin_block / 64 << "];\n";
        o << "    const Acc *const partials = (const Acc *)p.ws_partials;\n";
        o << "    const idx_t nparts = " << nparts_expr << ";\n";
        o << "    for (idx_t group = blockIdx.x; group < p.nrows; group += gridDim.x) {\n";
        // The single-term sums read an element whose position comes from the inputs alone: those
        // loads (an index, then the element it names -- two round trips to memory) are issued
        // before the partials are folded instead of after.
        bool early = !gathers.empty();
        {
            std::vector<int> it;
            for (const Gather &ga : gathers) it.push_back(ga.index_value);
            const std::vector<char> ineed = needed(it);
            for (size_t n = 0; n < ineed.size(); n++) if (ineed[n] && g.nodes[n].kind == NodeKind::Reduce && real_reduce((int)n)) early = false;
        }
        if (early) emit_group_epilogue(level, group_out_ops, gathers, "        ", nullptr, nullptr, 1);
        o << "        const Acc *const gpart = partials + (size_t)group * (size_t)nparts;\n";
        o << "        Acc tot = Acc_identity();\n";
        if (inflight <= 1) {
            o << "        for (idx_t i = lane; i < nparts; i += " << fin_block << ") tot = Acc_combine()(tot, gpart[i]);\n";
        } else {
            o << "        for (idx_t i0 = lane; i0 < nparts; i0 += " << fin_block * inflight << ") {\n";
            o << "            Acc part_[" << inflight << "];\n";
            o << "            #pragma unroll\n            for (int u = 0; u < " << inflight << "; ++u) {\n";
            o << "                const idx_t i = i0 + (idx_t)u * " << fin_block << ";\n";
            o << "                part_[u] = Acc_identity();\n";
            o << "                if (i < nparts) part_[u] = gpart[i];\n";
            o << "            }\n";
            o << "            #pragma unroll\n            for (int u = 0; u < " << inflight << "; ++u) tot = Acc_combine()(tot, part_[u]);\n";
            o << "        }\n";
        }
        o << "        tot = ewf_block_reduce<" << fin_block / 64 << ">(tot, Acc_combine(), sm_fin, lane);\n";
        o << "        if (lane != 0) continue;\n";
        emit_group_epilogue(level, group_out_ops, gathers, "        ", nullptr, nullptr, early ? 2 : 0);
        o << "    }\n}\n";
    }

    // The same fold when reductions over the kept axes follow (a mean over the rows of per-row
    // values): one workgroup takes all groups, a wavefront per group in turn -- its lanes fold the
    // group's partials, its first lane evaluates the group's values, stores the per-group outputs
    // and adds the group's term to the wavefront's running cross-group accumulator -- and at the
    // end folds the wavefronts' accumulators in a fixed order and writes the final outputs.  One
    // launch instead of a fold per group followed by a kernel for the second reduction.
    // With few partials per group (`per_thread`) a thread takes a whole group instead: all groups
    // are then in flight at once, which matters when there are hundreds of them.
    int emit_finish_all(const std::vector<int> &level, const std::vector<int> &group_out_ops, const std::vector<int> &final_out_ops,
                        const std::string &nparts_expr, int64_t ngroups, const std::vector<Gather> &gathers, bool per_thread)
    {
        const int waves = (int)std::min<int64_t>(16, std::max<int64_t>(1, per_thread ? (ngroups + 63) / 64 : ngroups));
        const int fb = waves * 64;
        o << "\n// folds the partials of every reduction group, then the groups' values, in a fixed order\n";
        o << "extern \"C\" __global__ void __launch_bounds__(" << fb << ") ewf_finish(const Params p)\n{\n";
        o << "    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;\n";
        o << "    (void)lane;\n";
        o << "    __shared__ AccX sm_accx[" << waves << "];\n";
        o << "    const Acc *const partials = (const Acc *)p.ws_partials;\n";
        o << "    const idx_t nparts = " << nparts_expr << ";\n";
        o << "    AccX totx = AccX_identity();\n";
        if (per_thread) o << "    for (idx_t group = threadIdx.x; group < p.nrows; group += " << fb << ") {\n";
        else o << "    for (idx_t group = wave; group < p.nrows; group += " << waves << ") {\n";
        bool early = !gathers.empty();
        {
            std::vector<int> it;
            for (const Gather &ga : gathers) it.push_back(ga.index_value);
            const std::vector<char> ineed = needed(it);
            for (size_t n = 0; n < ineed.size(); n++) if (ineed[n] && g.nodes[n].kind == NodeKind::Reduce && real_reduce((int)n)) early = false;
        }
        epilogue_extra_targets.clear();
        for (int n : red.cross_nodes) epilogue_extra_targets.push_back(g.nodes[n].args[0]);
        if (early) emit_group_epilogue(level, group_out_ops, gathers, "        ", nullptr, nullptr, 1);
        if (per_thread) o << "        const Acc *const gpart = partials + (size_t)group;          // partial i of a group at [i][group]\n";
        else o << "        const Acc *const gpart = partials + (size_t)group * (size_t)nparts;\n";
        o << "        Acc tot = Acc_identity();\n";
        if (per_thread) {
            // eight partials in flight per thread, folded in their order
            o << "        for (idx_t i0 = 0; i0 < nparts; i0 += 8) {\n";
            o << "            Acc part_[8];\n";
            o << "            #pragma unroll\n            for (int u = 0; u < 8; ++u) {\n";
            o << "                part_[u] = Acc_identity();\n";
            o << "                if (i0 + u < nparts) part_[u] = gpart[(size_t)(i0 + u) * (size_t)p.nrows];\n";
            o << "            }\n";
            o << "            #pragma unroll\n            for (int u = 0; u < 8; ++u) tot = Acc_combine()(tot, part_[u]);\n";
            o << "        }\n";
        } else {
            o << "        for (idx_t i = lane; i < nparts; i += 64) tot = Acc_combine()(tot, gpart[i]);\n";
            o << "        tot = ewf_wave_reduce(tot, Acc_combine());\n";
            o << "        if (lane != 0) continue;\n";
        }
        emit_group_epilogue(level, group_out_ops, gathers, "        ", nullptr, nullptr, early ? 2 : 0);
        emit_cross_partial("        ", "totx = AccX_combine()(totx, ax);");
        epilogue_extra_targets.clear();
        o << "    }\n";
        if (per_thread) {
            o << "    totx = ewf_block_reduce<" << waves << ">(totx, AccX_combine(), sm_accx, (int)threadIdx.x);\n";
            o << "    if (threadIdx.x == 0) {\n";
            o << "        const AccX tot = totx;\n";
        } else {
            o << "    if (lane == 0) sm_accx[wave] = totx;\n";
            o << "    __syncthreads();\n";
            o << "    if (threadIdx.x == 0) {\n";
            o << "        AccX tot = sm_accx[0];\n";
            o << "        for (int w = 1; w < " << waves << "; ++w) tot = AccX_combine()(tot, sm_accx[w]);\n";
        }
        emit_results("tot", red.cross_nodes, "        ");
        std::vector<int> tg;
        for (int k : final_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> need = needed(tg);
        EmitCtx fx;
        fx.input = [&](int k) { return "ewf_in(((const " + std::string(ctype(c.ops[k].storage)) + " *)p." + opname(k) + ")[0])"; };
        fx.coord = [&](int) { return std::string("0"); };
        emit_values(need, fx, "        ");
        for (int k : final_out_ops) {
            const Operand &op = c.ops[k];
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << "        ((" << ctype(op.storage) << " *)p." << opname(k) << ")[0] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
        }
        o << "    }\n}\n";
        return fb;
    }

    // What one thread does with the folded accumulator `tot` of reduction group `group`: the
    // results of the reductions, the single-term sums it reads itself, the values computed from
    // them, and the stores of the per-group outputs.
    // A caller that already has the group's coordinates passes their names in `coords` (one per
    // dimension, read for the kept ones) and spares the divisions; `store`, when given, emits
    // the store of output operand k instead of the plain scalar store.
    typedef std::function<void(int k, const std::string &value, const std::string &ind)> GroupStore;
    std::vector<char> epilogue_based;          // operands whose base pointer the epilogue has declared
    std::vector<int> epilogue_extra_targets;   // values the epilogue computes besides the group outputs
    void emit_group_epilogue(const std::vector<int> &level, const std::vector<int> &group_out_ops,
                             const std::vector<Gather> &gathers, const std::string &ind,
                             const std::vector<std::string> *coords = nullptr, const GroupStore *store = nullptr, int part = 0)
    {
        // part 1: the group's coordinates and the single-term sums only (nothing that needs `tot`);
        // part 2: the rest, in a scope that part 1 was emitted into; 0: both
        std::vector<int> all_dims;
        for (int d = 0; d < R; d++) all_dims.push_back(d);
        if (part == 2) {}
        else if (coords) {
            for (int d = 0; d < R; d++)
                o << ind << "const idx_t o" << d << " = " << (c.reduced[d] ? std::string("0") : (*coords)[d]) << ";\n";
        }
        else {
            o << ind << "idx_t g_ = group;\n";
            for (int d = R - 1; d >= 0; d--) {
                if (c.reduced[d]) { o << ind << "const idx_t o" << d << " = 0;\n"; continue; }
                bool last_kept = true;
                for (int d2 = d - 1; d2 >= 0; d2--) if (!c.reduced[d2]) last_kept = false;
                if (!last_kept) o << ind << "const idx_t o" << d << " = g_ % p.ext[" << d << "]; g_ /= p.ext[" << d << "];\n";
                else o << ind << "const idx_t o" << d << " = g_;\n";
            }
            o << ind << "(void)g_;\n";
        }
        if (part != 2) for (int d = 0; d < R; d++) o << ind << "(void)o" << d << ";\n";
        if (part != 1) emit_results("tot", level, ind);
        std::vector<int> gt;
        for (int k : group_out_ops) gt.push_back(g.outputs[c.ops[k].index].value);
        for (int n : epilogue_extra_targets) gt.push_back(n);
        std::vector<char> gneed = needed(gt);
        EmitCtx gx;
        gx.input = [&](int k) { return "ewf_in(q_" + opname(k) + "[0])"; };
        gx.coord = [&](int d) { return "o" + std::to_string(d); };
        if (part != 2) epilogue_based.assign(c.ops.size(), 0);
        std::vector<char> &based = epilogue_based;
        auto base_once = [&](int k) {
            if (based[k]) return;
            based[k] = 1;
            emit_base(k, all_dims, ind);
        };
        if (!gathers.empty()) {
            std::vector<int> it;
            for (const Gather &ga : gathers) it.push_back(ga.index_value);
            std::vector<char> ineed = needed(it);
            if (part != 2) {
                for (int k : inputs_of(ineed)) base_once(k);
                emit_values(ineed, gx, ind);
            }
            for (size_t n = 0; n < ineed.size(); n++) if (ineed[n]) gneed[n] = 0;
            for (const Gather &ga : gathers) {
                if (part == 2) break;
                base_once(ga.input);
                const std::string nm = opname(ga.input);
                o << ind << "float r" << ga.node << ";\n" << ind << "{\n";
                o << ind << "    const int t_ = v" << ga.index_value << ";\n";
                o << ind << "    const bool in_ = t_ >= 0 && t_ < p.ext[" << ga.cdim << "];\n";
                o << ind << "    const float x_ = ewf_in(q_" << nm << "[(idx_t)(in_ ? t_ : 0) * p.st_" << nm << "[" << ga.cdim << "]]);\n";
                o << ind << "    r" << ga.node << " = in_ ? x_ + 0.0f : 0.0f;\n" << ind << "}\n";
            }
        }
        if (part == 1) return;
        for (int k : inputs_of(gneed)) base_once(k);
        emit_values(gneed, gx, ind);
        for (int k : group_out_ops) {
            const Operand &op = c.ops[k];
            int v = g.outputs[op.index].value;
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            base_once(k);
            const std::string value = std::string(cv) + "(v" + std::to_string(v) + ")";
            if (store) (*store)(k, value, ind);
            else o << ind << "q_" << opname(k) << "[0] = " << value << ";\n";
        }
    }

    // One row's contribution to the cross-row reductions (the value of their arguments for this
    // row, already emitted as v<n>) goes to partials[row].
    void emit_cross_partial(const std::string &ind, const std::string &sink = "partials[row] = ax;")
    {
        o << ind << "AccX ax = AccX_identity();\n";
        for (size_t i = 0; i < red.cross_nodes.size(); i++) {
            if (shared_slot(red.cross_nodes, i) >= 0) continue;
            const Node &nd = g.nodes[red.cross_nodes[i]];
            o << ind << "ax.a" << i << " = v" << nd.args[0] << ";\n";
            if (nd.op == kRSumExpShifted) o << ind << "ax.b" << i << " = 1.0f;\n";
            if (nd.op == kRSumSqCentred) o << ind << "ax.n" << i << " = 1.0f;\n" << ind << "ax.b" << i << " = 0.0f;\n";
            if (nd.op == EWF_RARGMAX)
                o << ind << "ax.i" << i << " = " << argmax_index(red.cross_nodes[i], [](int d) { return "o" + std::to_string(d); }) << ";\n";
        }
        o << ind << sink << "\n";
    }

    // The per-row values are folded by a second, single-workgroup kernel: ordered by the kernel
    // boundary, deterministic, and free of atomics.
    // Returns the workgroup size of that kernel (more threads, and several loads in flight per
    // thread, when there are thousands of rows).
    int emit_cross_finish(const std::vector<int> &final_out_ops, int64_t nrows)
    {
        const int fb = nrows > 2048 ? 1024 : 256;
        const int inflight = (int)std::min<int64_t>(8, std::max<int64_t>(1, (nrows + fb - 1) / fb));
        o << "\nextern \"C\" __global__ void __launch_bounds__(" << fb << ") ewf_finish(const Params p)\n{\n";
        o << "    const int tid = threadIdx.x;\n";
        o << "    __shared__ AccX sm_accx[" << fb / 64 << "];\n";
        o << "    const AccX *const partials = (const AccX *)p.ws_partials;\n";
        o << "    AccX tot = AccX_identity();\n";
        o << "    for (idx_t i0 = tid; i0 < p.nrows; i0 += " << fb * inflight << ") {\n";
        o << "        AccX part_[" << inflight << "];\n";
        o << "        #pragma unroll\n        for (int u = 0; u < " << inflight << "; ++u) {\n";
        o << "            const idx_t i = i0 + (idx_t)u * " << fb << ";\n";
        o << "            part_[u] = AccX_identity();\n";
        o << "            if (i < p.nrows) part_[u] = partials[i];\n";
        o << "        }\n";
        o << "        #pragma unroll\n        for (int u = 0; u < " << inflight << "; ++u) tot = AccX_combine()(tot, part_[u]);\n";
        o << "    }\n";
        o << "    tot = ewf_block_reduce<" << fb / 64 << ">(tot, AccX_combine(), sm_accx, tid);\n";
        o << "    if (tid == 0) {\n";
        emit_results("tot", red.cross_nodes, "        ");
        std::vector<int> tg;
        for (int k : final_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> need = needed(tg);
        EmitCtx fx;
        fx.input = [&](int k) { return "ewf_in(((const " + std::string(ctype(c.ops[k].storage)) + " *)p." + opname(k) + ")[0])"; };
        fx.coord = [&](int) { return std::string("0"); };
        emit_values(need, fx, "        ");
        for (int k : final_out_ops) {
            const Operand &op = c.ops[k];
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << "        ((" << ctype(op.storage) << " *)p." << opname(k) << ")[0] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
        }
        o << "    }\n}\n";
        return fb;
    }

    ewf_status gen_tile(bool with_reduce);
    ewf_status gen_lane();
    ewf_status gen_row();
    ewf_status gen_col();
};


inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace ewf

#endif  // EWF_GEN_H
