// HIP source generator.
//
// One kernel per (expression, storage types, canonical layout class, vector width, index
// width); extents, strides and run-time scalars are kernel arguments so that a new shape of
// the same class reuses the compiled code (paper section 5.3 argues for passing such
// information at run time instead of baking it into generated modules; section 2.2.3
// describes per-node code generation, which here becomes per-fused-expression).
//
// Three kernel skeletons, all written for 64-lane wavefronts:
//   Tile        element-wise: grid-stride loop over n-d tiles; per tile every thread issues
//               all of its wide loads, then evaluates the scalar graph in registers, then
//               stores.
//   TileReduce  Tile plus per-thread accumulators; one tile never leaves its reduction
//               group; every wavefront stores one partial result to the workspace and a
//               second small kernel folds the partials of each group in a fixed order.
//   Row         one workgroup owns whole rows of the innermost (reduced) dimension, keeps
//               the row in registers and runs the chained reduction levels over it
//               (row max, then sum of exp(x - max), ...); an optional cross-row reduction
//               goes through the workspace and the same kind of second kernel.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <functional>
#include <sstream>

#include "ewf_internal.h"

namespace ewf {

// ------------------------------------------------------------------ parameter block

void ParamLayout::add(ParamField::Type t, const std::string &name, int count)
{
    // count 0 declares a scalar member, any other count an array of that many
    fields.push_back({t, name, count});
}

int ParamLayout::find(const std::string &name) const
{
    for (size_t i = 0; i < fields.size(); i++) if (fields[i].name == name) return (int)i;
    return -1;
}

static size_t field_size(ParamField::Type t) { return (t == ParamField::Ptr || t == ParamField::I64) ? 8 : 4; }

std::string ParamLayout::declare(const std::string &struct_name, bool) const
{
    std::ostringstream o;
    o << "struct " << struct_name << " {\n";
    for (const ParamField &f : fields) {
        const char *ty = f.type == ParamField::Ptr ? "void *" : f.type == ParamField::I64 ? "long long " :
                         f.type == ParamField::I32 ? "int " : "float ";
        o << "    " << ty << f.name;
        if (f.count > 0) o << "[" << f.count << "]";
        o << ";\n";
    }
    o << "};\n";
    return o.str();
}

static void finish_layout(ParamLayout &L)
{
    size_t off = 0, maxal = 4;
    L.offsets.clear();
    for (const ParamField &f : L.fields) {
        size_t sz = field_size(f.type);
        maxal = std::max(maxal, sz);
        off = (off + sz - 1) / sz * sz;
        L.offsets.push_back(off);
        off += sz * (size_t)std::max(1, f.count);
    }
    L.size = (off + maxal - 1) / maxal * maxal;
}

// ------------------------------------------------------------------ helpers

static const char *ctype(ewf_dtype t) { return t == EWF_F16 ? "ewf_half" : t == EWF_I32 ? "int" : "float"; }
static const char *vtype_c(ewf_dtype t) { return t == EWF_I32 ? "int" : "float"; }
static int isz(ewf_dtype t) { return t == EWF_F16 ? 2 : 4; }

static std::string f32_literal(double v)
{
    float f = (float)v;
    uint32_t b;
    memcpy(&b, &f, 4);
    char buf[64];
    snprintf(buf, sizeof buf, "ewf_bits_f32(0x%08xu)", b);
    return buf;
}

static std::string i32_literal(double v)
{
    int64_t w = (int64_t)v;
    uint32_t b = (uint32_t)(uint64_t)w;
    char buf[64];
    snprintf(buf, sizeof buf, "((int)0x%08xu)", b);
    return buf;
}

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
        std::vector<char> direct(N, 0);
        for (const OutputDecl &od : g.outputs) direct[od.value] = 1;
        for (int n = N - 1; n >= 0; n--) {
            if (!direct[n]) continue;
            const Node &nd = g.nodes[n];
            if (nd.kind == NodeKind::Reduce && nd.op == EWF_RSUM && nd.vtype == EWF_F32 && real_reduce(n)) continue;
            for (int a = 0; a < nd.nargs; a++) direct[nd.args[a]] = 1;
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
            const int fl = (e.auto_math && e.math_flavour == 1 && sum_only[n]) ? 2 : e.math_flavour;
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
                case EWF_EXP: rhs = std::string(M) + "::exp(" + a0 + ")"; break;
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
            b += (op == EWF_RARGMAX || op == kRSumExpShifted) ? 8 : 4;
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
            case EWF_RARGMAX: {
                std::string ia = "x.i" + std::to_string(i), ib = "y.i" + std::to_string(i);
                if (isint) {
                    o << "        { const bool t = (" << b << " > " << a << ") || (" << b << " == " << a << " && " << ib << " < " << ia << ");\n";
                } else {
                    // NaN ranks above every number; equal keys keep the lower index
                    o << "        { const bool gt = (" << b << " > " << a << ") || (" << b << " != " << b << " && " << a << " == " << a << ");\n"
                      << "          const bool eq = (" << b << " == " << a << ") || (" << b << " != " << b << " && " << a << " != " << a << ");\n"
                      << "          const bool t = gt || (eq && " << ib << " < " << ia << ");\n";
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
            else o << ind << "const " << vtype_c(nd.vtype) << " r" << nodes[i] << " = " << acc << ".a" << (sh >= 0 ? sh : (int)i) << ";\n";
        }
    }

    // Folds one element into every slot of the accumulator `acc` (slot-wise, no temporaries).
    // With `ascending` the caller guarantees that one thread meets the indices of an arg-max
    // in increasing order: a later element then replaces the running maximum only when it is
    // strictly greater (or the first NaN), and the index comparison falls away.  The
    // identity index (no element taken yet) must then be resolved by emit_first_index.
    void emit_accumulate(const std::string &acc, const std::vector<int> &nodes,
                         const std::function<std::string(int)> &argmax_index, const std::string &ind,
                         bool ascending = false)
    {
        for (size_t i = 0; i < nodes.size(); i++) {
            if (shared_slot(nodes, i) >= 0) continue;
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
            case EWF_RARGMAX: {
                std::string ia = acc + ".i" + std::to_string(i);
                std::string ib = "(int)(" + argmax_index(nodes[i]) + ")";
                if (ascending && isint) {
                    o << ind << "{ const bool t = " << v << " > " << a << ";\n";
                } else if (ascending) {
                    // greater, or the first NaN; a NaN already held stays
                    o << ind << "{ const bool t = !(" << v << " <= " << a << ") && (" << a << " == " << a << ");\n";
                } else if (isint) {
                    o << ind << "{ const bool t = (" << v << " > " << a << ") || (" << v << " == " << a << " && " << ib << " < " << ia << ");\n";
                } else {
                    o << ind << "{ const bool gt = (" << v << " > " << a << ") || (" << v << " != " << v << " && " << a << " == " << a << ");\n"
                      << ind << "  const bool eq = (" << v << " == " << a << ") || (" << v << " != " << v << " && " << a << " != " << a << ");\n"
                      << ind << "  const bool t = gt || (eq && " << ib << " < " << ia << ");\n";
                }
                o << ind << "  " << a << " = t ? " << v << " : " << a << "; " << ia << " = t ? " << ib << " : " << ia << "; }\n";
                break;
            }
            }
        }
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

    int argmax_canon_dim(int node) const
    {
        const Node &nd = g.nodes[node];
        for (int d = 0; d < g.ndim; d++) if (nd.axes & (1u << d)) return c.orig_of_axis[d];
        return -1;
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
        emit_group_epilogue(level, group_out_ops, gathers, "        ");
        o << "    }\n}\n";
    }

    // What one thread does with the folded accumulator `tot` of reduction group `group`: the
    // results of the reductions, the single-term sums it reads itself, the values computed from
    // them, and the stores of the per-group outputs.
    void emit_group_epilogue(const std::vector<int> &level, const std::vector<int> &group_out_ops,
                             const std::vector<Gather> &gathers, const std::string &ind)
    {
        std::vector<int> all_dims;
        for (int d = 0; d < R; d++) all_dims.push_back(d);
        o << ind << "idx_t g_ = group;\n";
        for (int d = R - 1; d >= 0; d--) {
            if (c.reduced[d]) { o << ind << "const idx_t o" << d << " = 0;\n"; continue; }
            bool last_kept = true;
            for (int d2 = d - 1; d2 >= 0; d2--) if (!c.reduced[d2]) last_kept = false;
            if (!last_kept) o << ind << "const idx_t o" << d << " = g_ % p.ext[" << d << "]; g_ /= p.ext[" << d << "];\n";
            else o << ind << "const idx_t o" << d << " = g_;\n";
        }
        for (int d = 0; d < R; d++) o << ind << "(void)o" << d << ";\n";
        o << ind << "(void)g_;\n";
        emit_results("tot", level, ind);
        std::vector<int> gt;
        for (int k : group_out_ops) gt.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> gneed = needed(gt);
        EmitCtx gx;
        gx.input = [&](int k) { return "ewf_in(q_" + opname(k) + "[0])"; };
        gx.coord = [&](int d) { return "o" + std::to_string(d); };
        std::vector<char> based(c.ops.size(), 0);
        auto base_once = [&](int k) {
            if (based[k]) return;
            based[k] = 1;
            emit_base(k, all_dims, ind);
        };
        if (!gathers.empty()) {
            std::vector<int> it;
            for (const Gather &ga : gathers) it.push_back(ga.index_value);
            std::vector<char> ineed = needed(it);
            for (int k : inputs_of(ineed)) base_once(k);
            emit_values(ineed, gx, ind);
            for (size_t n = 0; n < ineed.size(); n++) if (ineed[n]) gneed[n] = 0;
            for (const Gather &ga : gathers) {
                base_once(ga.input);
                const std::string nm = opname(ga.input);
                o << ind << "float r" << ga.node << ";\n" << ind << "{\n";
                o << ind << "    const int t_ = v" << ga.index_value << ";\n";
                o << ind << "    const bool in_ = t_ >= 0 && t_ < p.ext[" << ga.cdim << "];\n";
                o << ind << "    const float x_ = ewf_in(q_" << nm << "[(idx_t)(in_ ? t_ : 0) * p.st_" << nm << "[" << ga.cdim << "]]);\n";
                o << ind << "    r" << ga.node << " = in_ ? x_ + 0.0f : 0.0f;\n" << ind << "}\n";
            }
        }
        for (int k : inputs_of(gneed)) base_once(k);
        emit_values(gneed, gx, ind);
        for (int k : group_out_ops) {
            const Operand &op = c.ops[k];
            int v = g.outputs[op.index].value;
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            base_once(k);
            o << ind << "q_" << opname(k) << "[0] = " << cv << "(v" << v << ");\n";
        }
    }

    ewf_status gen_tile(bool with_reduce);
    ewf_status gen_row();
    ewf_status gen_col();
};

// =========================================================================================
// Tile / TileReduce

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

ewf_status Gen::gen_tile(bool with_reduce)
{
    // vectors in flight per thread: two for streaming expressions; one when the expression is
    // heavy in transcendental operations, where registers (occupancy) matter more
    int heavy = 0;
    for (size_t n = 0; n < g.nodes.size(); n++) {
        if (live[n] && g.nodes[n].kind == NodeKind::Reduce && g.nodes[n].op == kRSumExpShifted) heavy += 1;
        if (!live[n] || g.nodes[n].kind != NodeKind::Apply) continue;
        switch (g.nodes[n].op) {
        case EWF_EXP: case EWF_LOG: case EWF_LOG1P: case EWF_TANH: case EWF_SIGMOID: case EWF_EXPM1: heavy += 1; break;
        case EWF_POW: heavy += 2; break;
        default: break;
        }
    }
    // small problems are latency-bound: one vector per thread and small workgroups, so that
    // every compute unit gets work and nobody loops
    const int64_t items = c.total / VEC;
    const bool small = items < (int64_t)256 * 512;
    const int U = e.opts.unroll > 0 ? e.opts.unroll : ((heavy >= 4 || small) ? 1 : 2);
    // arithmetic-heavy expressions run best with larger workgroups (measured on the 21-op
    // float16 workload: 512 threads beat 256 by 4-8 %), streaming ones with 256
    int block = heavy >= 4 ? 512 : 256;
    if (small) { block = 64; while (block < 256 && items / block > 512) block *= 2; }
    if (e.opts.block_threads > 0) block = e.opts.block_threads;
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");

    // ---- outputs by role
    std::vector<int> ew_out_ops, group_out_ops;        // operand numbers
    const int nin = g.ninputs;
    for (size_t k = nin; k < c.ops.size(); k++) {
        const Node &v = g.nodes[g.outputs[c.ops[k].index].value];
        const int vn = g.outputs[c.ops[k].index].value;
        bool group = with_reduce && ((v.bcast & red.axes) == red.axes);
        if (with_reduce && red.edepth[vn] >= 1 && !group) return fail("an output depends on a reduction and varies along the reduced axes; only the row-resident class covers that");
        (group ? group_out_ops : ew_out_ops).push_back((int)k);
    }

    // ---- tile shape: innermost dimensions first, never across a group boundary
    int64_t T[kMaxDims];
    for (int d = 0; d < kMaxDims; d++) T[d] = 1;
    // several trips per tile amortise the per-tile address set-up; small problems keep
    // one trip per tile so that they still spread over the whole chip
    const int64_t one_trip = (int64_t)block * VEC * U;
    int64_t target = one_trip * 4;
    if (!with_reduce) {
        // ... but never so few tiles that the last round of workgroups leaves much of the
        // chip idle: at least about 32 tiles per compute unit (measured on four float16 input
        // streams: 3328 tiles of 15680 elements ran at 5.5 TB/s, 8192 of 6272 at 6.2-6.4)
        const int64_t want_tiles = (int64_t)32 * device_cu_count();
        target = std::max(one_trip, std::min(target, c.total / want_tiles));
    }
    if (e.opts.tile_elems > 0) target = e.opts.tile_elems;
    {
        int64_t rem = target;
        for (int d = R - 1; d >= 0 && rem > 1; d--) {
            if (with_reduce && !c.reduced[d]) break;
            if (c.extent[d] <= rem) { T[d] = c.extent[d]; rem /= T[d]; continue; }
            int64_t n = ceil_div(c.extent[d], rem);
            int64_t t = ceil_div(c.extent[d], n);
            if (d == R - 1) t = ceil_div(t, VEC) * VEC;
            T[d] = t;
            break;
        }
    }
    // ---- permuted operands: stage through LDS
    // An operand whose own fastest dimension is not the output's would be read with one
    // narrow access per element.  Instead the workgroup reads the operand's part of the tile
    // along the operand's fastest dimension with wide accesses, scatters it into an LDS copy
    // of the tile laid out in the output's order, and the compute phase reads it back with
    // one wide LDS access per vector.  The tile is shaped so that both sides see long runs.
    std::vector<int> staged;                           // operand numbers
    std::vector<int> sdims;                            // dims ordered by the staged operand's stride
    int VS = 1;
    if (!with_reduce && !e.opts.no_lds_staging && c.total >= 65536 && R >= 2) {
        for (int k = 0; k < nin && staged.empty(); k++) {
            const Operand &op = c.ops[k];
            if (op.access != Access::Gather) continue;
            bool full = true; int s0 = -1;
            for (int d = 0; d < R; d++) { if (op.stride[d] == 0) full = false; if (op.stride[d] == 1) s0 = d; }
            if (!full || s0 < 0 || c.extent[s0] < 16) continue;
            staged.push_back(k);
        }
    }
    if (!staged.empty()) {
        const Operand &S = c.ops[staged[0]];
        const int szS = isz(S.storage);
        for (int d = 0; d < R; d++) sdims.push_back(d);
        std::sort(sdims.begin(), sdims.end(), [&](int a, int b) { return S.stride[a] < S.stride[b]; });
        // other permuted operands that walk memory in the same order share the tile
        for (int k = 0; k < nin; k++) {
            if (k == staged[0] || c.ops[k].access != Access::Gather || isz(c.ops[k].storage) != szS) continue;
            bool same = true;
            for (int d = 0; d < R; d++) if (c.ops[k].stride[d] != S.stride[d]) same = false;
            if (same) staged.push_back(k);
        }
        // 64 KiB of LDS per staged operand (two workgroups per compute unit): room for runs along
        // the output's order that are whole cache lines
        const int64_t budget = (e.opts.tile_elems > 0 ? e.opts.tile_elems : 65536 / szS);
        for (int d = 0; d < kMaxDims; d++) T[d] = 1;
        // runs of at least 128 bytes along the staged operand's memory order
        int64_t need_run = 128 / szS;
        for (size_t i = 0; i < sdims.size() && need_run > 1; i++) {
            int d = sdims[i];
            T[d] = std::min<int64_t>(c.extent[d], need_run);
            if (T[d] < c.extent[d]) break;
            if (i + 1 < sdims.size() && S.stride[sdims[i + 1]] != S.stride[d] * c.extent[d]) break;
            need_run = ceil_div(need_run, T[d]);
        }
        // then the longest runs along the output's order that the LDS budget allows
        for (int d = R - 1; d >= 0; d--) {
            int64_t others = 1;
            for (int d2 = 0; d2 < R; d2++) if (d2 != d) others *= T[d2];
            int64_t cap = std::max<int64_t>(1, budget / others);
            int64_t t = std::max<int64_t>(T[d], std::min<int64_t>(c.extent[d], cap));
            if (t < c.extent[d]) {
                // prefer a split whose runs in the contiguous operands are whole 128-byte lines
                // (a line shared by two tiles is fetched twice: the tiles run on different dies),
                // then an even split of the dimension, then the larger tile
                int64_t run = 1;                          // elements of a run below this dimension
                for (int d2 = d + 1; d2 < R; d2++) run *= T[d2];
                int64_t best_q = t; int best_score = -1;
                for (int64_t q = t; q >= std::max<int64_t>(T[d], t / 2 + 1); q--) {
                    int score = ((q * run * szS) % 128 == 0 ? 2 : 0) + (c.extent[d] % q == 0 ? 1 : 0);
                    if (score > best_score) { best_score = score; best_q = q; }
                }
                t = best_q;
            }
            if (d == R - 1) t = std::max<int64_t>(VEC, t / VEC * VEC);
            T[d] = t;
            if (t < c.extent[d]) break;
        }
        // vector width on the staging side
        const int s0 = sdims[0];
        VS = 16 / szS;
        auto vs_ok = [&](int v) {
            if (T[s0] % v || c.extent[s0] % v) return false;
            for (int k : staged) {
                if (c.ops[k].addr % (uint64_t)(v * szS)) return false;
                for (int d = 0; d < R; d++) if (d != s0 && c.ops[k].stride[d] % v) return false;
            }
            return true;
        };
        while (VS > 1 && !vs_ok(VS)) VS /= 2;
    }
    auto is_staged = [&](int k) { return std::find(staged.begin(), staged.end(), k) != staged.end(); };
    if (!staged.empty() && e.opts.block_threads <= 0) {
        // two workgroups of twelve wavefronts share a compute unit when the staged tile takes about
        // half its LDS (measured on both readings of the float16 stress workload: 768 threads 89-90 us,
        // 512 threads 93-94 us, 1024 threads 101-108 us)
        int64_t te = 1;
        for (int d = 0; d < R; d++) te *= T[d];
        if (te * isz(c.ops[staged[0]].storage) > 40 * 1024) block = 768;
    }
    p.block = block;

    // LDS copy of the tile: the output's order, with a few padding elements after every run
    // of the staged operand's fastest dimension so that the scattering writes of one
    // wavefront (lanes that differ along that dimension) spread over the LDS banks.
    int64_t LS[kMaxDims], LSP[kMaxDims];
    int64_t lds_pad = 0, lds_elems = 0;
    { int64_t acc_ = 1; for (int d = R - 1; d >= 0; d--) { LS[d] = acc_; LSP[d] = acc_; acc_ *= T[d]; } lds_elems = acc_; }
    if (!staged.empty()) {
        const int s0 = sdims[0];
        const int szS = isz(c.ops[staged[0]].storage);
        std::vector<int> st;
        for (int d : sdims) if (T[d] > 1) st.push_back(d);
        auto conflicts = [&](int64_t pad) {
            // passes one scattered write of a wavefront needs: the LDS has 32 banks of 4 bytes
            // and takes the 64 lanes as two halves; a half needs as many passes as the largest
            // number of distinct words that fall into one bank
            int total = 0;
            for (int half = 0; half < 2; half++) {
                std::map<int64_t, std::vector<int64_t>> bank;
                for (int lane = half * 32; lane < half * 32 + 32; lane++) {
                    int64_t j = (int64_t)lane * VS, addr = 0;
                    for (size_t i = 0; i < st.size(); i++) {
                        int d = st[i];
                        int64_t cd = (i + 1 < st.size()) ? j % T[d] : j; j /= T[d];
                        int64_t ls = LS[d];
                        if (LS[d] >= LS[s0]) ls = LS[d] / LS[s0] * (LS[s0] + pad);
                        addr += cd * ls;
                    }
                    int64_t word = addr * szS / 4;
                    auto &v = bank[word % 32];
                    if (std::find(v.begin(), v.end(), word) == v.end()) v.push_back(word);
                }
                size_t worst = 0;
                for (auto &kv : bank) worst = std::max(worst, kv.second.size());
                total += (int)worst;
            }
            return total;
        };
        // fewest passes first; among equals the padding that keeps the widest aligned reads on
        // the consuming side (16 bytes, then 8), then the smallest
        auto read_bytes = [&](int64_t pad) { int64_t b = pad * szS; return b % 16 == 0 ? 16 : b % 8 == 0 ? 8 : 4; };
        int best = conflicts(0);
        for (int64_t pad = 4 / szS; pad * szS <= 64; pad += 4 / szS) {
            int cf = conflicts(pad);
            if (cf < best || (cf == best && read_bytes(pad) > read_bytes(lds_pad))) { best = cf; lds_pad = pad; }
        }
        for (int d = 0; d < R; d++) if (LS[d] >= LS[s0]) LSP[d] = LS[d] / LS[s0] * (LS[s0] + lds_pad);
        lds_elems = lds_elems / LS[s0] * (LS[s0] + lds_pad);
    }

    int64_t TE = 1;
    for (int d = 0; d < R; d++) TE *= T[d];
    const int64_t step = (int64_t)block * VEC * U;
    int fin_block_out = 64;
    int64_t ntile[kMaxDims], ntiles = 1;
    for (int d = 0; d < R; d++) { ntile[d] = ceil_div(c.extent[d], T[d]); ntiles *= ntile[d]; p.tile[d] = T[d]; }
    if (TE > ((int64_t)1 << 30) || ntiles >= ((int64_t)1 << 31) - 1) return fail("tile count out of range");

    std::vector<int> tiled;                            // dims with T > 1, innermost first
    for (int d = R - 1; d >= 0; d--) if (T[d] > 1) tiled.push_back(d);
    const int in_d = R - 1;

    // ---- what to evaluate per element
    std::vector<int> targets;
    for (int k : ew_out_ops) targets.push_back(g.outputs[c.ops[k].index].value);
    // Sums with one non-zero term are left to the second kernel, which reads that element
    // itself (as long as something else remains to be accumulated here).
    std::vector<int> level;
    std::vector<Gather> gathers;
    if (with_reduce) {
        for (int n : red.level_nodes) {
            Gather ga;
            if (match_gather(n, ga) && g.nodes[n].axes == red.axes && c.reduced[ga.cdim]) gathers.push_back(ga);
            else level.push_back(n);
        }
        if (level.empty()) { level = red.level_nodes; gathers.clear(); }
    }
    for (int n : level) targets.push_back(g.nodes[n].args[0]);
    // One thread meets the elements of a tile in increasing order of the linear index; when the
    // tile extends along the arg-max axis only, that is increasing order of the arg-max index.
    bool ascending = with_reduce && tiled.size() <= 1;
    for (int n : level)
        if (g.nodes[n].op == EWF_RARGMAX && !tiled.empty() && argmax_canon_dim(n) != tiled[0]) ascending = false;
    std::vector<char> need = needed(targets);
    std::vector<int> used_inputs = inputs_of(need);

    emit_header(block);
    build_layout();
    if (with_reduce) emit_acc_struct("Acc", level);
    std::vector<int> all_dims;
    for (int d = 0; d < R; d++) all_dims.push_back(d);
    std::vector<int> load_ops;                         // operand numbers read per element
    for (int k : used_inputs) load_ops.push_back(k);

    // what one trip of a thread holds in registers between its loads and its arithmetic
    o << "struct Item {\n    bool ok[" << U << "];\n    int L[" << U << "];\n";
    for (int d : tiled) o << "    int c" << d << "[" << U << "];\n";
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        if (op.access == Access::Splat && !is_staged(k)) o << "    " << ctype(op.storage) << " x_" << opname(k) << "[" << U << "];\n";
        else o << "    ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
    }
    o << "};\n";

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    std::string ind = "        ";
    // When every reduction group is a single tile the workgroup holds the whole group: it folds
    // its wavefronts through LDS and writes the results itself -- one launch, no workspace.
    bool one_tile = with_reduce;
    for (int d = 0; d < R; d++) if (c.reduced[d] && ntile[d] != 1) one_tile = false;
    if (with_reduce && !one_tile) o << "    Acc *const partials = (Acc *)p.ws_partials;\n";
    if (one_tile) o << "    __shared__ Acc sm_one[EWF_NWAVES];\n";
    for (int k : staged)
        o << "    __shared__ __attribute__((aligned(16))) " << ctype(c.ops[k].storage) << " lds_" << opname(k) << "[" << lds_elems << "];\n";
    // tiles are numbered in canonical (memory) order so that the workgroups resident at any
    // moment stream neighbouring addresses
    // Optional die-aware numbering: workgroups are handed to the eight accelerator dies
    // round-robin and each die has its own L2; with xcd_remap workgroup w takes tile
    // (w mod 8) * ceil(ntiles / 8) + w / 8, so the tiles in flight on one die are neighbours
    // in memory.  Off by default: measured slower on the streaming workloads (eight distant
    // streams instead of one; 145 us against 136 us on the bias + ReLU + channel-sum workload).
    const bool xcd_remap = e.opts.xcd_remap && ntiles >= 64;
    if (xcd_remap) {
        o << "    const idx_t chunk_ = (p.ntiles + 7) / 8;\n";
        o << "    for (idx_t wg_ = blockIdx.x; wg_ < chunk_ * 8; wg_ += gridDim.x) {\n";
        o << "        const idx_t tile = (wg_ & 7) * chunk_ + (wg_ >> 3);\n";
        o << "        if (tile >= p.ntiles) continue;\n";
    } else {
        o << "    for (idx_t tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {\n";
    }
    o << "        idx_t t_ = tile;\n";
    for (int d = R - 1; d >= 0; d--) {
        if (d > 0) o << "        const idx_t ti" << d << " = ewf_uniform(t_ % p.ntile[" << d << "]); t_ /= p.ntile[" << d << "];\n";
        else o << "        const idx_t ti0 = ewf_uniform(t_);\n";
        o << "        const idx_t o" << d << " = ti" << d << " * " << T[d] << ";\n";
    }
    if (with_reduce) o << "        Acc acc = Acc_identity();\n";
    for (int k : load_ops) emit_base(k, all_dims, ind);
    for (int k : ew_out_ops) emit_base(k, all_dims, ind);

    // Offset of an item inside the tile.  Two things are decided here from the strides the
    // plan was made for (they are part of the plan's key, and the choice is part of the
    // generated text): products whose factors are below 2^24 use the full-rate 24-bit multiply
    // (the 32-bit one runs at a quarter of the rate), and an operand that walks the tile's
    // dimensions (nearly) contiguously starts from the item's linear index in the tile and adds
    // only the dimensions where its stride differs from the tile's own pitch.
    int64_t pitch[kMaxDims];                               // linear index step of one unit along d
    { int64_t acc_ = 1; for (int d : tiled) { pitch[d] = acc_; acc_ *= T[d]; } }
    auto product = [&](const std::string &coord, const std::string &factor, int64_t factor_value) {
        if (c.byte32 && factor_value >= 0 && factor_value < ((int64_t)1 << 24))
            return "ewf_mul24(" + coord + ", " + factor + ")";
        return "(ioff_t)" + coord + " * (ioff_t)(" + factor + ")";
    };
    if (!staged.empty()) {
        const int s0 = sdims[0];
        o << ind << "for (int J0 = 0; J0 < " << TE << "; J0 += " << (int64_t)block * VS << ") {\n";
        o << ind << "    int j_ = J0 + tid * " << VS << ";\n";
        o << ind << "    bool k_ = j_ < " << TE << ";\n";
        o << ind << "    int lm_ = 0; ioff_t g_ = 0;\n";
        std::vector<int> st;                           // staged-order dims with T > 1
        for (int d : sdims) if (T[d] > 1) st.push_back(d);
        for (size_t i = 0; i < st.size(); i++) {
            int d = st[i];
            o << ind << "    { const int c_ = " << (i + 1 < st.size() ? "j_ % " + std::to_string(T[d]) + "; j_ /= " + std::to_string(T[d]) : std::string("j_")) << ";\n";
            if (c.extent[d] % T[d]) o << ind << "      k_ = k_ && (o" << d << " + c_ < p.ext[" << d << "]);\n";
            o << ind << "      lm_ += c_ * " << LSP[d] << ";\n";
            if (d == s0) o << ind << "      g_ += (ioff_t)c_; }\n";
            else o << ind << "      g_ += " << product("c_", "p.st_" + opname(staged[0]) + "[" + std::to_string(d) + "]", c.ops[staged[0]].stride[d]) << "; }\n";
        }
        o << ind << "    if (k_) {\n";
        for (int k : staged) {
            const Operand &op = c.ops[k];
            // a staged operand is read exactly once through these wide loads: stream it past the
            // caches under the same rule as the unit-stride operands
            int64_t fp_ = isz(op.storage);
            for (int d = 0; d < R; d++) if (op.stride[d] != 0) fp_ *= c.extent[d];
            const bool nt_ = e.opts.streaming == 1 || (e.opts.streaming == 0 && fp_ >= ((int64_t)32 << 20));
            o << ind << "        { const ewf_vec<" << ctype(op.storage) << ", " << VS << "> v_ = " << (nt_ ? "ewf_ld_nt<" : "ewf_ld<")
              << ctype(op.storage) << ", " << VS << ">(ewf_at(q_" << opname(k) << ", g_));\n";
            o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < " << VS << "; ++e_) lds_" << opname(k) << "[lm_ + e_ * " << LSP[s0] << "] = v_.e[e_]; }\n";
        }
        o << ind << "    }\n";
        o << ind << "}\n";
        o << ind << "__syncthreads();\n";
    }
    const bool looped = TE > step;
    const std::string ind0 = ind;

    auto offset_expr = [&](int k, bool skip_inner) {
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        bool linear = !skip_inner && !tiled.empty() && tiled[0] == in_d && op.stride[in_d] == 1;
        for (int d : tiled) if (op.stride[d] < pitch[d]) linear = false;
        std::string s;
        if (linear) {
            s = "(ioff_t)it.L[u]";
            for (int d : tiled) {
                if (op.stride[d] == pitch[d]) continue;
                s += " + " + product("it.c" + std::to_string(d) + "[u]", "p.st_" + nm + "[" + std::to_string(d) + "] - " + std::to_string(pitch[d]),
                                     op.stride[d] - pitch[d]);
            }
            return s;
        }
        for (int d : tiled) {
            if (op.stride[d] == 0) continue;
            if (d == in_d && skip_inner) continue;
            if (!s.empty()) s += " + ";
            if (d == in_d && op.stride[d] == 1) s += "(ioff_t)it.c" + std::to_string(d) + "[u]";
            else s += product("it.c" + std::to_string(d) + "[u]", "p.st_" + nm + "[" + std::to_string(d) + "]", op.stride[d]);
        }
        return s.empty() ? std::string("(ioff_t)0") : s;
    };

    // The text of one trip in three pieces: coordinates and mask of the thread's items (A), its
    // loads (B), and the arithmetic with accumulation and stores (C).  They are assembled
    // either as two local functions (so that the next trip's loads can be issued ahead of the
    // current trip's arithmetic) or, when there is no such prefetch, as one function that keeps
    // loads and arithmetic under a single mask: the values then never cross a branch, which
    // otherwise costs a register copy per loaded word.
    auto capture = [&](const std::function<void()> &emit) {
        const std::string before = o.str();
        o.str("");
        emit();
        const std::string text = o.str();
        o.str("");
        o << before;
        return text;
    };
    const std::string ind2 = ind + "    ";
    const std::string text_a = capture([&]() {
        o << ind2 << "    const int L = L0 + (u * EWF_BLOCK + tid) * EWF_VEC;\n";
        o << ind2 << "    it.L[u] = L;\n";
        o << ind2 << "    bool k_ = L < " << TE << ";\n";
        if (!tiled.empty()) {
            o << ind2 << "    int l_ = L;\n";
            for (size_t i = 0; i < tiled.size(); i++) {
                int d = tiled[i];
                if (i + 1 < tiled.size()) o << ind2 << "    it.c" << d << "[u] = l_ % " << T[d] << "; l_ /= " << T[d] << ";\n";
                else o << ind2 << "    it.c" << d << "[u] = l_;\n";
                if (c.extent[d] % T[d]) o << ind2 << "    k_ = k_ && (o" << d << " + it.c" << d << "[u] < p.ext[" << d << "]);\n";
            }
        }
    });
    const std::string text_b = capture([&]() {
        const std::string &ind = ind2;
        for (int k : load_ops) {
            const Operand &op = c.ops[k];
            std::string nm = opname(k);
            if (is_staged(k)) {
                // padded position of the item in the LDS copy; wide pieces as far as the padding
                // keeps them aligned
                const int s0 = sdims[0];
                const int szk = isz(op.storage);
                int piece = VEC;                               // elements per LDS access
                while (piece > 1 && ((lds_pad * szk) % (piece * szk) != 0 || piece * szk > 16)) piece /= 2;
                std::string pos = lds_pad ? "(L + (L / " + std::to_string(LS[s0]) + ") * " + std::to_string(lds_pad) + ")" : std::string("L");
                if (piece == VEC)
                    o << ind << "        it.x_" << nm << "[u] = ewf_ld<" << ctype(op.storage) << ", EWF_VEC>(&lds_" << nm << "[" << pos << "]);\n";
                else
                    o << ind << "        _Pragma(\"unroll\") for (int i_ = 0; i_ < " << VEC / piece << "; ++i_) ((ewf_vec<" << ctype(op.storage) << ", " << piece
                      << "> *)&it.x_" << nm << "[u])[i_] = ewf_ld<" << ctype(op.storage) << ", " << piece << ">(&lds_" << nm << "[" << pos << " + i_ * " << piece << "]);\n";
            }
            else if (op.access == Access::Vector)
                o << ind << "        it.x_" << nm << "[u] = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << offset_expr(k, false) << "));\n";
            else if (op.access == Access::Splat)
                o << ind << "        it.x_" << nm << "[u] = *ewf_at(q_" << nm << ", " << offset_expr(k, true) << ");\n";
            else {
                o << ind << "        { const ioff_t b_ = " << offset_expr(k, false) << ";\n";
                o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) it.x_" << nm << "[u].e[e_] = *ewf_at(q_" << nm
                  << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm << "[" << in_d << "]); }\n";
            }
        }
    });
    const std::string text_c = capture([&]() {
        const std::string &ind = ind2;
        for (int k : ew_out_ops) o << ind << "    ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
        o << ind << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        EmitCtx cx;
        cx.input = [&](int k) {
            const Operand &op = c.ops[k];
            if (op.access == Access::Splat && !is_staged(k)) return "ewf_in(it.x_" + opname(k) + "[u])";
            if (op.storage == EWF_F16 && VEC >= 2) return "ewf_in_h(it.x_" + opname(k) + "[u], e_)";
            return "ewf_in(it.x_" + opname(k) + "[u].e[e_])";
        };
        cx.coord = [&](int d) {
            std::string s = "o" + std::to_string(d);
            if (T[d] > 1) s += " + it.c" + std::to_string(d) + "[u]";
            if (d == in_d) s += " + e_";
            return s;
        };
        emit_values(need, cx, ind + "        ");
        if (with_reduce)
            emit_accumulate("acc", level, [&](int node) { return cx.coord(argmax_canon_dim(node)); }, ind + "        ", ascending);
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            int v = g.outputs[op.index].value;
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << ind << "        y_" << opname(k) << ".e[e_] = " << cv << "(v" << v << ");\n";
        }
        o << ind << "    }\n";
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            std::string nm = opname(k);
            if (op.access == Access::Vector)
                o << ind << "    " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << offset_expr(k, false) << "), y_" << nm << ");\n";
            else {
                o << ind << "    { const ioff_t b_ = " << offset_expr(k, op.access == Access::Splat) << ";\n";
                o << ind << "      _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) *ewf_at(q_" << nm << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm
                  << "[" << in_d << "]) = y_" << nm << ".e[e_]; }\n";
            }
        }
    });

    const bool prefetch = looped && !(e.opts.no_prefetch == 1 || (heavy >= 4 && e.opts.no_prefetch == 0));
    if (prefetch) {
        o << ind << "auto load_item = [&](const int L0, Item &it) {\n";
        o << ind2 << "#pragma unroll\n" << ind2 << "for (int u = 0; u < " << U << "; ++u) {\n";
        o << text_a;
        o << ind2 << "    it.ok[u] = k_;\n";
        o << ind2 << "    if (k_) {\n" << text_b << ind2 << "    }\n" << ind2 << "}\n";
        o << ind << "};\n";
        o << ind << "auto eval_item = [&](const Item &it) {\n";
        o << ind2 << "#pragma unroll\n" << ind2 << "for (int u = 0; u < " << U << "; ++u) {\n";
        o << ind2 << "    if (!it.ok[u]) continue;\n";
        o << text_c;
        o << ind2 << "}\n";
        o << ind << "};\n";
        // the next trip's loads are issued before the current trip is evaluated, so that
        // arithmetic and memory latency overlap inside a wavefront as well as between wavefronts
        o << ind << "{\n";
        o << ind << "    Item cur, nxt;\n";
        o << ind << "    load_item(0, cur);\n";
        o << ind << "    for (int L0 = 0; L0 < " << TE << "; L0 += " << step << ") {\n";
        o << ind << "        const bool more = L0 + " << step << " < " << TE << ";\n";
        o << ind << "        if (more) load_item(L0 + " << step << ", nxt);\n";
        o << ind << "        eval_item(cur);\n";
        o << ind << "        if (more) cur = nxt;\n";
        o << ind << "    }\n";
        o << ind << "}\n";
    } else {
        o << ind << "auto run_item = [&](const int L0) {\n";
        o << ind2 << "Item it;\n";
        o << ind2 << "#pragma unroll\n" << ind2 << "for (int u = 0; u < " << U << "; ++u) {\n";
        o << text_a;
        o << ind2 << "    if (!k_) continue;\n";
        o << text_b << text_c;
        o << ind2 << "}\n";
        o << ind << "};\n";
        if (!looped) o << ind << "run_item(0);\n";
        else o << ind << "for (int L0 = 0; L0 < " << TE << "; L0 += " << step << ") run_item(L0);\n";
    }
    if (!staged.empty()) o << ind << "__syncthreads();\n";

    if (with_reduce) {
        // Every wavefront folds its own lanes with cross-lane moves and stores one partial:
        // no LDS, no barrier, no atomic -- the waves of a workgroup never wait for each other
        // and the kernel streams like a copy.  A second, tiny kernel folds the partials of a
        // group in a fixed order (deterministic, and ordered by the kernel boundary alone).
        if (ascending) {
            // a thread's first element of the tile is item tid of the first trip
            std::string first = "(idx_t)0", has = "tid * EWF_VEC < " + std::to_string(TE);
            if (!tiled.empty()) {
                const std::string d = std::to_string(tiled[0]);
                first = "o" + d + " + tid * EWF_VEC";
                has += " && o" + d + " + tid * EWF_VEC < p.ext[" + d + "]";
            } else {
                for (int n : level) if (g.nodes[n].op == EWF_RARGMAX) first = "o" + std::to_string(argmax_canon_dim(n));
            }
            emit_first_index("acc", level, has, first, ind);
        }
        o << ind << "idx_t group = 0, slot = 0;\n";
        for (int d = 0; d < R; d++) {
            if (c.reduced[d]) o << ind << "slot = slot * p.ntile[" << d << "] + ti" << d << ";\n";
            else o << ind << "group = group * p.ext[" << d << "] + o" << d << ";\n";
        }
        if (one_tile) {
            o << ind << "(void)slot;\n";
            o << ind << "acc = ewf_block_reduce<EWF_NWAVES>(acc, Acc_combine(), sm_one, tid);\n";
            o << ind << "if (tid == 0) {\n";
            o << ind << "    const Acc tot = acc;\n";
            emit_group_epilogue(level, group_out_ops, gathers, ind + "    ");
            o << ind << "}\n";
        } else {
            o << ind << "acc = ewf_wave_reduce(acc, Acc_combine());\n";
            o << ind << "if ((tid & 63) == 0) partials[((size_t)group * (size_t)p.nslots + (size_t)slot) * EWF_NWAVES + (tid >> 6)] = acc;\n";
        }
    }
    o << "    }\n}\n";

    if (with_reduce && !one_tile) {
        // one workgroup per group: a wavefront when a group has few partials, four otherwise
        int64_t nparts_host = (int64_t)(block / 64);
        for (int d = 0; d < R; d++) if (c.reduced[d]) nparts_host *= ntile[d];
        // (1024 threads and eight partials in flight per thread when there are thousands: a total
        // over a large tensor is one group, and its finish is otherwise a chain of dependent loads)
        const int fin_block = nparts_host > 4096 ? 1024 : nparts_host > 256 ? 256 : 64;
        fin_block_out = fin_block;
        const int inflight = (int)std::min<int64_t>(8, std::max<int64_t>(1, ceil_div(nparts_host, fin_block)));
        emit_finish_lanes(level, group_out_ops, "p.nslots * EWF_NWAVES", fin_block, inflight, gathers);
    }

    // ---- launch geometry and argument block
    int64_t cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : (int64_t)1 << 22;
    p.grid = std::max<int64_t>(1, xcd_remap ? std::min(ceil_div(ntiles, 8) * 8, std::max<int64_t>(8, cap / 8 * 8)) : std::min(ntiles, cap));
    p.lds_bytes = 0;
    p.staged = (int)staged.size();
    for (int k : staged) p.lds_bytes += (int)(lds_elems * isz(c.ops[k].storage));
    int64_t ngroups = 1, nslots = 1;
    for (int d = 0; d < R; d++) { if (c.reduced[d]) nslots *= ntile[d]; else ngroups *= c.extent[d]; }
    p.workspace_bytes = 0;
    p.finish_grid = 0;
    if (with_reduce && !one_tile) {
        if (ngroups >= ((int64_t)1 << 31) || nslots >= ((int64_t)1 << 31)) return fail("too many reduction groups");
        p.workspace_bytes = (size_t)ngroups * (size_t)nslots * (size_t)(block / 64) * acc_bytes(level);
        p.finish_grid = std::min<int64_t>(ngroups, (int64_t)1 << 20);
        p.finish_block = fin_block_out;
    }
    p.args.assign(p.layout.size, 0);
    auto put_idx = [&](const std::string &name, int i, int64_t v) {
        int f = p.layout.find(name);
        size_t off = p.layout.offsets[f];
        if (c.idx64) memcpy(&p.args[off + 8 * (size_t)i], &v, 8);
        else { int32_t w = (int32_t)v; memcpy(&p.args[off + 4 * (size_t)i], &w, 4); }
    };
    for (int d = 0; d < R; d++) { put_idx("ext", d, c.extent[d]); put_idx("ntile", d, ntile[d]); }
    put_idx("ntiles", 0, ntiles);
    put_idx("nrows", 0, ngroups);
    put_idx("nslots", 0, nslots);
    for (size_t k = 0; k < c.ops.size(); k++)
        for (int d = 0; d < R; d++) put_idx("st_" + opname((int)k), d, c.ops[k].stride[d]);
    p.source = o.str();
    return EWF_OK;
}

// =========================================================================================
// Row

ewf_status Gen::gen_row()
{
    const int in_d = R - 1;
    const int64_t cols = c.extent[in_d];
    int block = e.opts.block_threads;
    if (block <= 0) {
        block = 256;
        while (block > 64 && cols <= (int64_t)(block / 2) * VEC * 2) block /= 2;
        while (block < 1024 && cols > (int64_t)block * VEC * 12) block *= 2;
    }
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");
    p.block = block;
    const int nin = g.ninputs;

    // ---- roles of the outputs
    std::vector<int> full_out_ops, group_out_ops, final_out_ops;
    for (size_t k = nin; k < c.ops.size(); k++) {
        int vn = g.outputs[c.ops[k].index].value;
        const Node &v = g.nodes[vn];
        if (after_cross[vn]) final_out_ops.push_back((int)k);
        else if ((v.bcast & red.axes) == red.axes) group_out_ops.push_back((int)k);
        else full_out_ops.push_back((int)k);
    }
    // ---- per-level targets
    const int D = red.max_depth;
    std::vector<std::vector<int>> lvl(D + 1);
    std::vector<std::vector<Gather>> gat(D + 1);
    for (int n : red.level_nodes) {
        Gather ga;
        if (match_gather(n, ga) && ga.cdim == in_d) gat[red.edepth[n]].push_back(ga);
        else lvl[red.edepth[n]].push_back(n);
    }

    // which inputs vary along the row and are read by some per-element computation
    std::vector<int> elem_targets;
    for (int l = 1; l <= D; l++) for (int n : lvl[l]) elem_targets.push_back(g.nodes[n].args[0]);
    for (int k : full_out_ops) elem_targets.push_back(g.outputs[c.ops[k].index].value);
    std::vector<char> eneed = needed(elem_targets);
    std::vector<int> row_ops, splat_ops;
    for (int k : inputs_of(eneed)) (c.ops[k].stride[in_d] != 0 ? row_ops : splat_ops).push_back(k);

    // ---- residency: keep the row in registers when it fits
    const int64_t per_iter = (int64_t)block * VEC;
    const int64_t NV = ceil_div(cols, per_iter);
    int regs = 0;
    for (int k : row_ops) regs += (int)NV * VEC * isz(c.ops[k].storage) / 4;
    const bool resident = NV <= 32 && regs <= 96;
    if (p.avoid_poor_rows && e.opts.split_rows != 2) {
        int64_t nr = 1;
        for (int d = 0; d < R - 1; d++) nr *= c.extent[d];
        // measured on [rows, cols] float32 softmax cross-entropy of 268 MB: rows held in registers
        // run at 5.3-5.5 TB/s up to 32768 columns but 4.1 TB/s at 65536 (64 registers per thread,
        // 1024 threads: one workgroup per compute unit), rows streamed once per level 2.7-3.4 TB/s;
        // split over workgroups 5.0-5.2 TB/s at any row length
        const bool too_long = !resident || regs > 48;
        if (too_long || (nr * 2 < device_cu_count() && cols >= 16384) || e.opts.split_rows == 1) {
            p.row_refused = true;
            return fail(too_long ? "a row does not fit the registers of a workgroup well: the row class would read it once per reduction level or run one workgroup per compute unit"
                                 : "too few rows for one workgroup per row to occupy the chip");
        }
    }
    const int U = resident ? (int)NV : (e.opts.unroll > 0 ? e.opts.unroll : 4);
    p.tile[in_d] = cols;
    {
        // When all rows can be resident on the chip at once there is no second round of
        // workgroups (whose tail would idle most of the chip): ask the compiler for the
        // register budget that lets that many wavefronts share a SIMD, if the row leaves
        // room for the arithmetic under it.
        int64_t nrows_ = 1;
        for (int d = 0; d < R - 1; d++) nrows_ *= c.extent[d];
        const int64_t wg_per_cu = ceil_div(nrows_, device_cu_count());
        const int64_t waves = ceil_div(wg_per_cu * (block / 64), 4);
        if (resident && !p.no_auto_occupancy && waves >= 2 && waves <= 8 && regs + 40 <= 512 / waves / 8 * 8) {
            auto_waves_per_simd = (int)waves;
            p.used_auto_occupancy = !(e.opts.waves_per_simd >= 1 && e.opts.waves_per_simd <= 8);
        }
    }

    emit_header(block);
    build_layout();
    for (int l = 1; l <= D; l++) if (!lvl[l].empty()) emit_acc_struct("Acc" + std::to_string(l), lvl[l]);
    const bool has_cross = !red.cross_nodes.empty();
    if (has_cross) emit_acc_struct("AccX", red.cross_nodes);

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    o << "    const idx_t cols = p.ext[" << in_d << "];\n";
    for (int l = 1; l <= D; l++) if (!lvl[l].empty()) o << "    __shared__ Acc" << l << " sm_acc" << l << "[EWF_NWAVES];\n";
    if (has_cross) o << "    AccX *const partials = (AccX *)p.ws_partials;\n";
    // one workgroup per row when the grid can hold them all: no loop, so nothing is hoisted
    // out of it into registers that the row needs
    int64_t nrows = 1;
    for (int d = 0; d < R - 1; d++) nrows *= c.extent[d];
    if (nrows >= ((int64_t)1 << 31) - 1) return fail("too many rows");
    const int64_t grid_cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : (int64_t)256 * 32;
    if (nrows <= grid_cap) o << "    if ((idx_t)blockIdx.x < p.nrows) {\n        const idx_t row = blockIdx.x;\n";
    else o << "    for (idx_t row = blockIdx.x; row < p.nrows; row += gridDim.x) {\n";
    o << "        idx_t t_ = row;\n";
    std::vector<int> outer;
    for (int d = R - 2; d >= 0; d--) {
        if (d > 0) o << "        const idx_t o" << d << " = ewf_uniform(t_ % p.ext[" << d << "]); t_ /= p.ext[" << d << "];\n";
        else o << "        const idx_t o0 = ewf_uniform(t_);\n";
    }
    for (int d = 0; d < R - 1; d++) outer.push_back(d);
    std::vector<int> based;
    auto base_once = [&](int k, const std::string &ind) {
        if (std::find(based.begin(), based.end(), k) != based.end()) return;
        based.push_back(k);
        emit_base(k, outer, ind);
    };
    for (int k : row_ops) base_once(k, "        ");
    for (int k : splat_ops) base_once(k, "        ");
    for (int k : full_out_ops) base_once(k, "        ");

    // the loop over the row: either over register-resident vectors or streaming chunks
    // The first NFULL steps of a resident row are in range for every thread of the
    // workgroup at this plan's row length: straight-line code there lets the compiler wait
    // for the loads one by one instead of for all of them.  (The row length is part of the
    // plan's key, and NFULL of the generated text, so the assumption travels with the code.)
    const int64_t NFULL = resident ? cols / per_iter : 0;
    auto open_pass = [&]() {
        if (resident) {
            o << "        #pragma unroll\n        for (int u = 0; u < " << U << "; ++u) {\n";
            o << "            const idx_t col = (idx_t)(u * EWF_BLOCK + tid) * EWF_VEC;\n";
            o << "            if (u >= " << NFULL << " && col >= cols) continue;\n";
        } else {
            o << "        for (idx_t c0 = 0; c0 < cols; c0 += " << (per_iter * U) << ") {\n";
            o << "        #pragma unroll\n        for (int u = 0; u < " << U << "; ++u) {\n";
            o << "            const idx_t col = c0 + (idx_t)(u * EWF_BLOCK + tid) * EWF_VEC;\n";
            o << "            if (col >= cols) continue;\n";
        }
    };
    auto close_pass = [&]() {
        o << "        }\n";
        if (!resident) o << "        }\n";
    };
    auto emit_row_load = [&](int k, const std::string &ind, const std::string &dst) {
        const Operand &op = c.ops[k];
        std::string nm = opname(k);
        if (op.access == Access::Vector)
            o << ind << dst << " = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col);\n";
        else
            o << ind << "_Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) " << dst << ".e[e_] = q_" << nm
              << "[(col + e_) * p.st_" << nm << "[" << in_d << "]];\n";
    };

    // values constant along the row come first: an index that a gather depends on is then
    // the first load to return, and the dependent read queues right behind the row
    std::vector<int> uniform_loaded = splat_ops;
    for (int l = 1; l <= D; l++)
        for (const Gather &ga : gat[l])
            for (int k : inputs_of(needed(std::vector<int>{ga.index_value})))
                if (std::find(uniform_loaded.begin(), uniform_loaded.end(), k) == uniform_loaded.end()) uniform_loaded.push_back(k);
    for (int k : uniform_loaded) {
        base_once(k, "        ");
        o << "        const " << ctype(c.ops[k].storage) << " g_" << opname(k) << " = ewf_ld_uniform(q_" << opname(k) << ");\n";
    }
    if (resident) {
        for (int k : row_ops) o << "        ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
        open_pass();
        for (int k : row_ops) emit_row_load(k, "            ", "x_" + opname(k) + "[u]");
        close_pass();
    }

    EmitCtx cx;
    cx.input = [&](int k) {
        if (c.ops[k].stride[in_d] == 0) return "ewf_in(g_" + opname(k) + ")";
        return resident ? "ewf_in(x_" + opname(k) + "[u].e[e_])" : "ewf_in(w_" + opname(k) + ".e[e_])";
    };
    cx.coord = [&](int d) {
        if (d == in_d) return std::string("col + e_");
        return "o" + std::to_string(d);
    };
    auto stream_loads = [&](const std::vector<char> &need) {
        if (resident) return;
        for (int k : inputs_of(need)) {
            if (c.ops[k].stride[in_d] == 0) continue;
            o << "            ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> w_" << opname(k) << ";\n";
            emit_row_load(k, "            ", "w_" + opname(k));
        }
    };

    // values constant along the row, evaluated by every thread (uniform addresses)
    EmitCtx ux;
    ux.input = [&](int k) { return "ewf_in(g_" + opname(k) + ")"; };
    ux.coord = [&](int d) { return d == in_d ? std::string("0") : "o" + std::to_string(d); };

    for (int l = 1; l <= D; l++) {
        for (const Gather &ga : gat[l]) {
            // issued ahead of the level's pass so that the element arrives under it
            std::vector<char> need = needed(std::vector<int>{ga.index_value});
            base_once(ga.input, "        ");
            const std::string nm = opname(ga.input);
            // keep the wait for the index behind every load already issued
            o << "        __builtin_amdgcn_sched_barrier(0);\n";
            o << "        float r" << ga.node << ";\n        {\n";
            emit_values(need, ux, "            ");
            // the read itself is unconditional (index clamped into the row) so that it is one
            // more load in flight, not a branch the wavefront has to wait behind
            o << "            const int t_ = v" << ga.index_value << ";\n";
            o << "            const bool in_ = t_ >= 0 && t_ < cols;\n";
            o << "            const float x_ = ewf_in(q_" << nm << "[(idx_t)(in_ ? t_ : 0)"
              << (c.ops[ga.input].stride[in_d] == 1 ? std::string("") : " * p.st_" + nm + "[" + std::to_string(in_d) + "]")
              << "]);\n";
            o << "            r" << ga.node << " = in_ ? x_ + 0.0f : 0.0f;\n        }\n";
        }
        if (lvl[l].empty()) continue;
        std::string an = "Acc" + std::to_string(l), av = "acc" + std::to_string(l);
        std::vector<int> tg;
        for (int n : lvl[l]) tg.push_back(g.nodes[n].args[0]);
        std::vector<char> need = needed(tg);
        o << "        " << an << " " << av << " = " << an << "_identity();\n";
        open_pass();
        stream_loads(need);
        o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        emit_values(need, cx, "                ");
        emit_accumulate(av, lvl[l], [&](int node) { return cx.coord(argmax_canon_dim(node)); }, "                ", true);
        o << "            }\n";
        close_pass();
        // every thread walks its columns in increasing order, starting at tid * EWF_VEC
        emit_first_index(av, lvl[l], "(idx_t)tid * EWF_VEC < cols", "tid * EWF_VEC", "        ");
        o << "        " << av << " = ewf_block_reduce<EWF_NWAVES>(" << av << ", " << an << "_combine(), sm_acc" << l << ", tid);\n";
        emit_results(av, lvl[l], "        ");
    }

    if (!full_out_ops.empty()) {
        std::vector<int> tg;
        for (int k : full_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> need = needed(tg);
        open_pass();
        stream_loads(need);
        for (int k : full_out_ops) o << "            ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
        o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        emit_values(need, cx, "                ");
        for (int k : full_out_ops) {
            const Operand &op = c.ops[k];
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << "                y_" << opname(k) << ".e[e_] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
        }
        o << "            }\n";
        for (int k : full_out_ops) {
            const Operand &op = c.ops[k];
            std::string nm = opname(k);
            if (op.access == Access::Vector)
                o << "            " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col, y_" << nm << ");\n";
            else
                o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) q_" << nm << "[(col + e_) * p.st_" << nm
                  << "[" << in_d << "]] = y_" << nm << ".e[e_];\n";
        }
        close_pass();
    }

    // per-row values: results of the reductions, the outputs derived from them, and the
    // arguments of cross-row reductions
    {
        std::vector<int> tg;
        for (int k : group_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        for (int n : red.cross_nodes) tg.push_back(g.nodes[n].args[0]);
        if (!tg.empty()) {
            std::vector<char> need = needed(tg);
            o << "        if (tid == 0) {\n";
            for (int k : inputs_of(need)) {
                if (std::find(uniform_loaded.begin(), uniform_loaded.end(), k) != uniform_loaded.end()) continue;
                base_once(k, "            ");
                o << "            const " << ctype(c.ops[k].storage) << " g_" << opname(k) << " = q_" << opname(k) << "[0];\n";
            }
            EmitCtx gx;
            gx.input = [&](int k) { return "ewf_in(g_" + opname(k) + ")"; };
            gx.coord = [&](int d) { return d == in_d ? std::string("0") : "o" + std::to_string(d); };
            emit_values(need, gx, "            ");
            for (int k : group_out_ops) {
                const Operand &op = c.ops[k];
                const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
                emit_base(k, outer, "            ");
                o << "            q_" << opname(k) << "[0] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
            }
            if (has_cross) {
                o << "            AccX ax = AccX_identity();\n";
                for (size_t i = 0; i < red.cross_nodes.size(); i++) {
                    if (shared_slot(red.cross_nodes, i) >= 0) continue;
                    const Node &nd = g.nodes[red.cross_nodes[i]];
                    o << "            ax.a" << i << " = v" << nd.args[0] << ";\n";
                    if (nd.op == kRSumExpShifted) o << "            ax.b" << i << " = 1.0f;\n";
                    if (nd.op == EWF_RARGMAX) {
                        int cd = argmax_canon_dim(red.cross_nodes[i]);
                        o << "            ax.i" << i << " = (int)(" << (cd < 0 ? std::string("0") : "o" + std::to_string(cd)) << ");\n";
                    }
                }
                o << "            partials[row] = ax;\n";
            }
            o << "        }\n";
        }
    }
    o << "    }\n";

    o << "}\n";
    if (has_cross) {
        // the per-row values are folded by a second, single-workgroup kernel: ordered by the
        // kernel boundary, deterministic, and free of atomics
        o << "\nextern \"C\" __global__ void __launch_bounds__(EWF_FIN_BLOCK) ewf_finish(const Params p)\n{\n";
        o << "    const int tid = threadIdx.x;\n";
        o << "    __shared__ AccX sm_accx[EWF_FIN_BLOCK / 64];\n";
        o << "    const AccX *const partials = (const AccX *)p.ws_partials;\n";
        o << "    AccX tot = AccX_identity();\n";
        o << "    for (idx_t i = tid; i < p.nrows; i += EWF_FIN_BLOCK) tot = AccX_combine()(tot, partials[i]);\n";
        o << "    tot = ewf_block_reduce<EWF_FIN_BLOCK / 64>(tot, AccX_combine(), sm_accx, tid);\n";
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
    }

    // ---- launch geometry and argument block
    p.grid = std::max<int64_t>(1, std::min(nrows, grid_cap));
    p.lds_bytes = 0;
    p.workspace_bytes = 0;
    p.finish_grid = 0;
    if (has_cross) {
        p.workspace_bytes = (size_t)nrows * acc_bytes(red.cross_nodes);
        p.finish_grid = 1;
        p.finish_block = 256;
    }
    p.args.assign(p.layout.size, 0);
    auto put_idx = [&](const std::string &name, int i, int64_t v) {
        int f = p.layout.find(name);
        size_t off = p.layout.offsets[f];
        if (c.idx64) memcpy(&p.args[off + 8 * (size_t)i], &v, 8);
        else { int32_t w = (int32_t)v; memcpy(&p.args[off + 4 * (size_t)i], &w, 4); }
    };
    for (int d = 0; d < R; d++) { put_idx("ext", d, c.extent[d]); put_idx("ntile", d, 1); }
    put_idx("ntiles", 0, nrows);
    put_idx("nrows", 0, nrows);
    put_idx("nslots", 0, 1);
    for (size_t k = 0; k < c.ops.size(); k++)
        for (int d = 0; d < R; d++) put_idx("st_" + opname((int)k), d, c.ops[k].stride[d]);
    p.source = o.str();
    return EWF_OK;
}

// =========================================================================================
// Col: reductions whose reduced axes are not the fastest-varying ones in memory
//
// The lanes of a wavefront lie along the innermost (kept) dimension, so loads stay wide and
// coalesced and every lane owns its own columns: no cross-lane step at all.  The rows of the
// innermost reduced dimension are spread over the wavefronts of the workgroup (and over
// several workgroups, "slots", when there are few columns); the per-wavefront results meet in
// LDS in a fixed order, one partial per column and slot goes to the workspace, and a second
// kernel folds the slots of each column in slot order.

ewf_status Gen::gen_col()
{
    const int in_d = R - 1;
    int dR = -1;                                       // innermost reduced dimension
    for (int d = R - 1; d >= 0; d--) if (c.reduced[d]) { dR = d; break; }
    if (dR < 0 || c.reduced[in_d]) return fail("column class needs a kept innermost dimension");
    const int nin = g.ninputs;
    int block = e.opts.block_threads > 0 ? e.opts.block_threads : 256;
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");
    p.block = block;

    // ---- outputs by role
    std::vector<int> ew_out_ops, group_out_ops;
    for (size_t k = nin; k < c.ops.size(); k++) {
        const int vn = g.outputs[c.ops[k].index].value;
        const Node &v = g.nodes[vn];
        bool group = (v.bcast & red.axes) == red.axes;
        if (red.edepth[vn] >= 1 && !group) return fail("an output depends on a reduction and varies along the reduced axes");
        (group ? group_out_ops : ew_out_ops).push_back((int)k);
    }
    const std::vector<int> &level = red.level_nodes;

    // ---- thread layout: TX lanes along the columns, TY groups of lanes along the rows
    const int64_t colvecs = c.extent[in_d] / VEC;
    int TX = 64;
    if (colvecs < 64) { TX = 1; while (TX < colvecs) TX *= 2; }
    const int TY = block / TX;
    const int64_t TK = std::min<int64_t>(c.extent[in_d], (int64_t)TX * VEC);   // columns per tile
    // rows in flight per thread: four for streaming expressions, fewer when the expression is
    // heavy in transcendental operations (registers) or the problem is small (spread it out)
    int heavy = 0;
    for (size_t n = 0; n < g.nodes.size(); n++) {
        if (!live[n] || g.nodes[n].kind != NodeKind::Apply) continue;
        switch (g.nodes[n].op) {
        case EWF_EXP: case EWF_LOG: case EWF_LOG1P: case EWF_TANH: case EWF_SIGMOID: case EWF_EXPM1: heavy += 1; break;
        case EWF_POW: case EWF_DIV: heavy += 2; break;
        default: break;
        }
    }
    const bool small = c.total / VEC < (int64_t)256 * 512;
    const int U = e.opts.unroll > 0 ? e.opts.unroll : small ? 1 : heavy >= 4 ? 2 : 4;
    int64_t T[kMaxDims];
    for (int d = 0; d < kMaxDims; d++) T[d] = 1;
    T[in_d] = TK;
    {
        // rows per tile: enough tiles to fill the chip, but whole trips of the workgroup
        int64_t other = ceil_div(c.extent[in_d], TK);
        for (int d = 0; d < R - 1; d++) if (d != dR) other *= c.extent[d];
        const int64_t want = (int64_t)16 * device_cu_count();
        int64_t slices = std::max<int64_t>(1, std::min(ceil_div(want, other), ceil_div(c.extent[dR], (int64_t)TY * U)));
        int64_t tr = ceil_div(c.extent[dR], slices);
        if (e.opts.tile_elems > 0) tr = std::max<int64_t>(1, e.opts.tile_elems / TK);
        T[dR] = std::min(c.extent[dR], tr);
    }
    const int64_t TR = T[dR];
    int64_t ntile[kMaxDims], ntiles = 1;
    for (int d = 0; d < R; d++) { ntile[d] = ceil_div(c.extent[d], T[d]); ntiles *= ntile[d]; p.tile[d] = T[d]; }
    if (ntiles >= ((int64_t)1 << 31) - 1 || TR >= ((int64_t)1 << 30)) return fail("tile count out of range");
    int64_t ngroups = 1, nslots = 1;
    for (int d = 0; d < R; d++) { if (c.reduced[d]) nslots *= ntile[d]; else ngroups *= c.extent[d]; }
    if (ngroups >= ((int64_t)1 << 31) || nslots >= ((int64_t)1 << 31) || ngroups * nslots >= ((int64_t)1 << 40))
        return fail("too many reduction groups");

    const bool fin_lanes = nslots > 16;
    const int fin_block = nslots > 256 ? 256 : 64;

    // ---- what to evaluate per element
    std::vector<int> targets;
    for (int k : ew_out_ops) targets.push_back(g.outputs[c.ops[k].index].value);
    for (int n : level) targets.push_back(g.nodes[n].args[0]);
    std::vector<char> need = needed(targets);
    std::vector<int> load_ops = inputs_of(need);

    emit_header(block);
    o << "#define EWF_TX " << TX << "\n#define EWF_TY " << TY << "\n";
    build_layout();
    emit_acc_struct("Acc", level);
    std::vector<int> all_dims;
    for (int d = 0; d < R; d++) all_dims.push_back(d);

    auto off_expr = [&](int k) {
        // offset of (row r_, column cc_) from the tile's origin
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        std::string s;
        if (op.stride[dR] != 0) s = "(ioff_t)r_ * (ioff_t)p.st_" + nm + "[" + std::to_string(dR) + "]";
        if (op.stride[in_d] != 0) {
            if (!s.empty()) s += " + ";
            s += op.stride[in_d] == 1 ? std::string("(ioff_t)cc_") : "(ioff_t)cc_ * (ioff_t)p.st_" + nm + "[" + std::to_string(in_d) + "]";
        }
        return s.empty() ? std::string("(ioff_t)0") : s;
    };

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    o << "    const int tx = tid & (EWF_TX - 1), ty = tid / EWF_TX;\n";
    o << "    Acc *const partials = (Acc *)p.ws_partials;\n";
    if (TY > 1) o << "    __shared__ Acc sm_col[(EWF_TY - 1) * EWF_TX * EWF_VEC];\n";
    o << "    for (idx_t tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {\n";
    o << "        idx_t t_ = tile;\n";
    for (int d = R - 1; d >= 0; d--) {
        if (d > 0) o << "        const idx_t ti" << d << " = ewf_uniform(t_ % p.ntile[" << d << "]); t_ /= p.ntile[" << d << "];\n";
        else o << "        const idx_t ti0 = ewf_uniform(t_);\n";
        o << "        const idx_t o" << d << " = ti" << d << " * " << T[d] << ";\n";
    }
    std::string ind = "        ";
    for (int k : load_ops) emit_base(k, all_dims, ind);
    for (int k : ew_out_ops) emit_base(k, all_dims, ind);
    o << ind << "const int cc_ = tx * EWF_VEC;\n";
    o << ind << "const bool colok_ = cc_ < " << TK << " && o" << in_d << " + cc_ < p.ext[" << in_d << "];\n";
    o << ind << "const int rows_ = (int)((p.ext[" << dR << "] - o" << dR << ") < " << TR << " ? (p.ext[" << dR << "] - o" << dR << ") : " << TR << ");\n";
    o << ind << "Acc acc[EWF_VEC];\n";
    o << ind << "_Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) acc[e_] = Acc_identity();\n";
    o << ind << "for (int r0_ = ty; r0_ < rows_; r0_ += EWF_TY * " << U << ") {\n";
    // loads of U rows, then their arithmetic
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        if (op.stride[in_d] == 0) o << ind << "    " << ctype(op.storage) << " x_" << opname(k) << "[" << U << "];\n";
        else o << ind << "    ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
    }
    o << ind << "    #pragma unroll\n" << ind << "    for (int u = 0; u < " << U << "; ++u) {\n";
    o << ind << "        const int r_ = r0_ + u * EWF_TY;\n";
    o << ind << "        if (!colok_ || r_ >= rows_) continue;\n";
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        if (op.stride[in_d] == 0)
            o << ind << "        x_" << nm << "[u] = *ewf_at(q_" << nm << ", " << off_expr(k) << ");\n";
        else if (op.access == Access::Vector)
            o << ind << "        x_" << nm << "[u] = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << off_expr(k) << "));\n";
        else {
            o << ind << "        { const ioff_t b_ = " << off_expr(k) << ";\n";
            o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) x_" << nm << "[u].e[e_] = *ewf_at(q_" << nm
              << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm << "[" << in_d << "]); }\n";
        }
    }
    o << ind << "    }\n";
    o << ind << "    #pragma unroll\n" << ind << "    for (int u = 0; u < " << U << "; ++u) {\n";
    o << ind << "        const int r_ = r0_ + u * EWF_TY;\n";
    o << ind << "        if (!colok_ || r_ >= rows_) continue;\n";
    for (int k : ew_out_ops) o << ind << "        ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
    o << ind << "        _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
    EmitCtx cx;
    cx.input = [&](int k) {
        const Operand &op = c.ops[k];
        if (op.stride[in_d] == 0) return "ewf_in(x_" + opname(k) + "[u])";
        if (op.storage == EWF_F16 && VEC >= 2) return "ewf_in_h(x_" + opname(k) + "[u], e_)";
        return "ewf_in(x_" + opname(k) + "[u].e[e_])";
    };
    cx.coord = [&](int d) {
        std::string s = "o" + std::to_string(d);
        if (d == dR) s += " + r_";
        if (d == in_d) s += " + cc_ + e_";
        return s;
    };
    emit_values(need, cx, ind + "            ");
    emit_accumulate("acc[e_]", level, [&](int node) { return cx.coord(argmax_canon_dim(node)); }, ind + "            ");
    for (int k : ew_out_ops) {
        const Operand &op = c.ops[k];
        const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
        o << ind << "            y_" << opname(k) << ".e[e_] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
    }
    o << ind << "        }\n";
    for (int k : ew_out_ops) {
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        if (op.access == Access::Vector)
            o << ind << "        " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << off_expr(k) << "), y_" << nm << ");\n";
        else {
            o << ind << "        { const ioff_t b_ = " << off_expr(k) << ";\n";
            o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) *ewf_at(q_" << nm << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm
              << "[" << in_d << "]) = y_" << nm << ".e[e_]; }\n";
        }
    }
    o << ind << "    }\n";
    o << ind << "}\n";
    // the row groups of the workgroup meet in LDS; group 0 folds them in order
    if (TY > 1) {
        o << ind << "if (ty > 0) { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) sm_col[((ty - 1) * EWF_TX + tx) * EWF_VEC + e_] = acc[e_]; }\n";
        o << ind << "__syncthreads();\n";
        o << ind << "if (ty == 0) {\n";
        o << ind << "    for (int w_ = 0; w_ < EWF_TY - 1; ++w_)\n";
        o << ind << "        _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) acc[e_] = Acc_combine()(acc[e_], sm_col[(w_ * EWF_TX + tx) * EWF_VEC + e_]);\n";
        o << ind << "}\n";
    }
    o << ind << "if (ty == 0 && colok_) {\n";
    o << ind << "    size_t group = 0, slot = 0;\n";
    for (int d = 0; d < R; d++) {
        if (c.reduced[d]) o << ind << "    slot = slot * (size_t)p.ntile[" << d << "] + (size_t)ti" << d << ";\n";
        else if (d == in_d) o << ind << "    group = group * (size_t)p.ext[" << d << "] + (size_t)(o" << d << " + cc_);\n";
        else o << ind << "    group = group * (size_t)p.ext[" << d << "] + (size_t)o" << d << ";\n";
    }
    if (fin_lanes) o << ind << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) partials[(group + e_) * (size_t)p.nslots + slot] = acc[e_];\n";
    else o << ind << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) partials[slot * (size_t)p.nrows + group + e_] = acc[e_];\n";
    o << ind << "}\n";
    if (TY > 1) o << ind << "__syncthreads();\n";
    o << "    }\n}\n";

    // ---- second kernel.  Many slots per column: the partials of a column are contiguous and a
    // workgroup's lanes walk them.  Few: one thread per column folds its slots in slot order.
    if (fin_lanes) emit_finish_lanes(level, group_out_ops, "p.nslots", fin_block,
                                     (int)std::min<int64_t>(8, std::max<int64_t>(1, ceil_div(nslots, fin_block))));
    else {
    o << "\nextern \"C\" __global__ void __launch_bounds__(256) ewf_finish(const Params p)\n{\n";
    o << "    const Acc *const partials = (const Acc *)p.ws_partials;\n";
    o << "    for (idx_t group = blockIdx.x * 256 + threadIdx.x; group < p.nrows; group += gridDim.x * 256) {\n";
    o << "        Acc tot = partials[group];\n";
    o << "        for (idx_t s_ = 1; s_ < p.nslots; ++s_) tot = Acc_combine()(tot, partials[(size_t)s_ * (size_t)p.nrows + (size_t)group]);\n";
    o << "        idx_t g_ = group;\n";
    for (int d = R - 1; d >= 0; d--) {
        if (c.reduced[d]) { o << "        const idx_t o" << d << " = 0;\n"; continue; }
        bool last_kept = true;
        for (int d2 = d - 1; d2 >= 0; d2--) if (!c.reduced[d2]) last_kept = false;
        if (!last_kept) o << "        const idx_t o" << d << " = g_ % p.ext[" << d << "]; g_ /= p.ext[" << d << "];\n";
        else o << "        const idx_t o" << d << " = g_;\n";
    }
    for (int d = 0; d < R; d++) o << "        (void)o" << d << ";\n";
    emit_results("tot", level, "        ");
    {
        std::vector<int> gt;
        for (int k : group_out_ops) gt.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> gneed = needed(gt);
        for (int k : inputs_of(gneed)) emit_base(k, all_dims, "        ");
        EmitCtx gx;
        gx.input = [&](int k) { return "ewf_in(q_" + opname(k) + "[0])"; };
        gx.coord = [&](int d) { return "o" + std::to_string(d); };
        emit_values(gneed, gx, "        ");
        for (int k : group_out_ops) {
            const Operand &op = c.ops[k];
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            emit_base(k, all_dims, "        ");
            o << "        q_" << opname(k) << "[0] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
        }
    }
    o << "    }\n}\n";
    }

    // ---- launch geometry and argument block
    int64_t cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : (int64_t)1 << 22;
    p.grid = std::max<int64_t>(1, std::min(ntiles, cap));
    p.lds_bytes = TY > 1 ? (int)((TY - 1) * TX * VEC * acc_bytes(level)) : 0;
    if (p.lds_bytes > 60 * 1024) return fail("too many reductions for one column kernel (LDS)");
    p.staged = 0;
    p.workspace_bytes = (size_t)ngroups * (size_t)nslots * acc_bytes(level);
    p.finish_grid = fin_lanes ? std::min<int64_t>(ngroups, (int64_t)1 << 20)
                              : std::max<int64_t>(1, std::min<int64_t>(ceil_div(ngroups, 256), (int64_t)1 << 16));
    p.finish_block = fin_lanes ? fin_block : 256;
    p.args.assign(p.layout.size, 0);
    auto put_idx = [&](const std::string &name, int i, int64_t v) {
        int f = p.layout.find(name);
        size_t off = p.layout.offsets[f];
        if (c.idx64) memcpy(&p.args[off + 8 * (size_t)i], &v, 8);
        else { int32_t w = (int32_t)v; memcpy(&p.args[off + 4 * (size_t)i], &w, 4); }
    };
    for (int d = 0; d < R; d++) { put_idx("ext", d, c.extent[d]); put_idx("ntile", d, ntile[d]); }
    put_idx("ntiles", 0, ntiles);
    put_idx("nrows", 0, ngroups);
    put_idx("nslots", 0, nslots);
    for (size_t k = 0; k < c.ops.size(); k++)
        for (int d = 0; d < R; d++) put_idx("st_" + opname((int)k), d, c.ops[k].stride[d]);
    p.source = o.str();
    return EWF_OK;
}

// =========================================================================================

ewf_status generate(const Exec &e, Plan &p)
{
    Gen gen(e, p);
    switch (p.kclass) {
    case KernelClass::Tile: return gen.gen_tile(false);
    case KernelClass::TileReduce: return gen.gen_tile(true);
    case KernelClass::Row: return gen.gen_row();
    case KernelClass::Col: return gen.gen_col();
    default: set_error("no kernel class"); return EWF_EUNSUPPORTED;
    }
}

}  // namespace ewf
