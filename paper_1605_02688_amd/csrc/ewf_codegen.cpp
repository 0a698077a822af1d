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
                bool is_target = std::find(targets.begin(), targets.end(), n) != targets.end();
                (void)is_target;
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
        const char *M = e.fast_math ? "ewf_fast" : "ewf_acc";
        for (size_t n = 0; n < need.size(); n++) {
            if (!need[n]) continue;
            const Node &nd = g.nodes[n];
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
                case EWF_POW: rhs = std::string(M) + "::pow(" + a0 + ", " + a1 + ")"; break;
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

    // Declares `struct <name>` with one slot per reduction in `nodes`, its identity and its
    // combine function.
    void emit_acc_struct(const std::string &name, const std::vector<int> &nodes)
    {
        o << "struct " << name << " {\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            const Node &nd = g.nodes[nodes[i]];
            const Node &arg = g.nodes[nd.args[0]];
            if (nd.op == EWF_RARGMAX) o << "    " << vtype_c(arg.vtype) << " a" << i << "; int i" << i << ";\n";
            else o << "    " << vtype_c(nd.vtype) << " a" << i << ";\n";
        }
        o << "};\n";
        o << "EWF_DEV " << name << " " << name << "_identity()\n{\n    " << name << " a;\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string id;
            switch (nd.op) {
            case EWF_RSUM: id = isint ? "0" : "0.0f"; break;
            case EWF_RPROD: id = isint ? "1" : "1.0f"; break;
            case EWF_RMAX: case EWF_RARGMAX: id = isint ? "(-2147483647 - 1)" : "ewf_bits_f32(0xff800000u)"; break;
            case EWF_RMIN: id = isint ? "2147483647" : "ewf_bits_f32(0x7f800000u)"; break;
            }
            o << "    a.a" << i << " = " << id << ";\n";
            if (nd.op == EWF_RARGMAX) o << "    a.i" << i << " = 2147483647;\n";
        }
        o << "    return a;\n}\n";
        o << "struct " << name << "_combine {\n    EWF_DEV " << name << " operator()(const " << name << " &x, const "
          << name << " &y) const\n    {\n        " << name << " r;\n";
        for (size_t i = 0; i < nodes.size(); i++) {
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string a = "x.a" + std::to_string(i), b = "y.a" + std::to_string(i);
            switch (nd.op) {
            case EWF_RSUM: o << "        r.a" << i << " = " << (isint ? "ewf_addi(" + a + ", " + b + ")" : a + " + " + b) << ";\n"; break;
            case EWF_RPROD: o << "        r.a" << i << " = " << (isint ? "ewf_muli(" + a + ", " + b + ")" : a + " * " + b) << ";\n"; break;
            case EWF_RMAX: o << "        r.a" << i << " = ewf_max(" << a << ", " << b << ");\n"; break;
            case EWF_RMIN: o << "        r.a" << i << " = ewf_min(" << a << ", " << b << ");\n"; break;
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
            if (nd.op == EWF_RARGMAX) o << ind << "const int r" << nodes[i] << " = " << acc << ".i" << i << ";\n";
            else o << ind << "const " << vtype_c(nd.vtype) << " r" << nodes[i] << " = " << acc << ".a" << i << ";\n";
        }
    }

    // Folds one element into every slot of the accumulator `acc` (slot-wise, no temporaries).
    void emit_accumulate(const std::string &acc, const std::vector<int> &nodes,
                         const std::function<std::string(int)> &argmax_index, const std::string &ind)
    {
        for (size_t i = 0; i < nodes.size(); i++) {
            const Node &nd = g.nodes[nodes[i]];
            const bool isint = g.nodes[nd.args[0]].vtype == EWF_I32;
            std::string a = acc + ".a" + std::to_string(i), v = "v" + std::to_string(nd.args[0]);
            switch (nd.op) {
            case EWF_RSUM: o << ind << a << " = " << (isint ? "ewf_addi(" + a + ", " + v + ")" : a + " + " + v) << ";\n"; break;
            case EWF_RPROD: o << ind << a << " = " << (isint ? "ewf_muli(" + a + ", " + v + ")" : a + " * " + v) << ";\n"; break;
            case EWF_RMAX: o << ind << a << " = ewf_max(" << a << ", " << v << ");\n"; break;
            case EWF_RMIN: o << ind << a << " = ewf_min(" << a << ", " << v << ");\n"; break;
            case EWF_RARGMAX: {
                std::string ia = acc + ".i" + std::to_string(i);
                std::string ib = "(int)(" + argmax_index(nodes[i]) + ")";
                if (isint) {
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
    }

    void build_layout()
    {
        ParamLayout &L = p.layout;
        L.fields.clear();
        const ParamField::Type IDX = c.idx64 ? ParamField::I64 : ParamField::I32;
        for (size_t k = 0; k < c.ops.size(); k++) L.add(ParamField::Ptr, opname((int)k), 0);
        L.add(ParamField::Ptr, "ws_counters", 0);
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

    ewf_status fail(const std::string &why)
    {
        set_error("%s", why.c_str());
        return EWF_EUNSUPPORTED;
    }

    ewf_status gen_tile(bool with_reduce);
    ewf_status gen_row();
};

// =========================================================================================
// Tile / TileReduce

static int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

ewf_status Gen::gen_tile(bool with_reduce)
{
    const int block = e.opts.block_threads > 0 ? e.opts.block_threads : 256;
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");
    const int U = e.opts.unroll > 0 ? e.opts.unroll : 2;
    p.block = block;

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
    int64_t target = (int64_t)block * VEC * U * (with_reduce ? 4 : 1);
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
    int64_t TE = 1;
    for (int d = 0; d < R; d++) TE *= T[d];
    const int64_t step = (int64_t)block * VEC * U;
    int64_t ntile[kMaxDims], ntiles = 1;
    for (int d = 0; d < R; d++) { ntile[d] = ceil_div(c.extent[d], T[d]); ntiles *= ntile[d]; p.tile[d] = T[d]; }
    if (TE > ((int64_t)1 << 30) || ntiles >= ((int64_t)1 << 31) - 1) return fail("tile count out of range");

    std::vector<int> tiled;                            // dims with T > 1, innermost first
    for (int d = R - 1; d >= 0; d--) if (T[d] > 1) tiled.push_back(d);
    const int in_d = R - 1;

    // ---- what to evaluate per element
    std::vector<int> targets;
    for (int k : ew_out_ops) targets.push_back(g.outputs[c.ops[k].index].value);
    std::vector<int> level = with_reduce ? red.level_nodes : std::vector<int>();
    for (int n : level) targets.push_back(g.nodes[n].args[0]);
    std::vector<char> need = needed(targets);
    std::vector<int> used_inputs = inputs_of(need);

    emit_header(block);
    build_layout();
    if (with_reduce) emit_acc_struct("Acc", level);

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    std::vector<int> all_dims;
    for (int d = 0; d < R; d++) all_dims.push_back(d);
    std::vector<int> load_ops;                         // operand numbers read per element
    for (int k : used_inputs) load_ops.push_back(k);
    std::string ind = "        ";
    if (with_reduce) o << "    Acc *const partials = (Acc *)p.ws_partials;\n";
    // tiles are numbered in canonical (memory) order so that the workgroups resident at any
    // moment stream neighbouring addresses
    o << "    for (idx_t tile = blockIdx.x; tile < p.ntiles; tile += gridDim.x) {\n";
    o << "        idx_t t_ = tile;\n";
    for (int d = R - 1; d >= 0; d--) {
        if (d > 0) o << "        const idx_t ti" << d << " = t_ % p.ntile[" << d << "]; t_ /= p.ntile[" << d << "];\n";
        else o << "        const idx_t ti0 = t_;\n";
        o << "        const idx_t o" << d << " = ti" << d << " * " << T[d] << ";\n";
    }
    if (with_reduce) o << "        Acc acc = Acc_identity();\n";
    for (int k : load_ops) emit_base(k, all_dims, ind);
    for (int k : ew_out_ops) emit_base(k, all_dims, ind);

    const bool looped = TE > step;
    const std::string ind0 = ind;
    if (looped) { o << ind << "for (int L0 = 0; L0 < " << TE << "; L0 += " << step << ") {\n"; ind += "    "; }
    else o << ind << "const int L0 = 0;\n";

    // phase A: coordinates, masks, loads
    o << ind << "bool ok[" << U << "];\n";
    for (int d : tiled) o << ind << "int c" << d << "[" << U << "];\n";
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        if (op.access == Access::Splat) o << ind << ctype(op.storage) << " x_" << opname(k) << "[" << U << "];\n";
        else o << ind << "ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
    }
    auto offset_expr = [&](int k, bool skip_inner) {
        const Operand &op = c.ops[k];
        std::string s;
        for (int d : tiled) {
            if (op.stride[d] == 0) continue;
            if (d == in_d && skip_inner) continue;
            if (!s.empty()) s += " + ";
            if (d == in_d && op.stride[d] == 1) s += "c" + std::to_string(d) + "[u]";
            else s += "(idx_t)c" + std::to_string(d) + "[u] * p.st_" + opname(k) + "[" + std::to_string(d) + "]";
        }
        return s.empty() ? std::string("0") : s;
    };
    o << ind << "#pragma unroll\n" << ind << "for (int u = 0; u < " << U << "; ++u) {\n";
    o << ind << "    const int L = L0 + (u * EWF_BLOCK + tid) * EWF_VEC;\n";
    o << ind << "    bool k_ = L < " << TE << ";\n";
    if (!tiled.empty()) {
        o << ind << "    int l_ = L;\n";
        for (size_t i = 0; i < tiled.size(); i++) {
            int d = tiled[i];
            if (i + 1 < tiled.size()) o << ind << "    c" << d << "[u] = l_ % " << T[d] << "; l_ /= " << T[d] << ";\n";
            else o << ind << "    c" << d << "[u] = l_;\n";
            o << ind << "    k_ = k_ && (o" << d << " + c" << d << "[u] < p.ext[" << d << "]);\n";
        }
    }
    o << ind << "    ok[u] = k_;\n";
    o << ind << "    if (k_) {\n";
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        std::string nm = opname(k);
        if (op.access == Access::Vector)
            o << ind << "        x_" << nm << "[u] = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + (" << offset_expr(k, false) << "));\n";
        else if (op.access == Access::Splat)
            o << ind << "        x_" << nm << "[u] = q_" << nm << "[" << offset_expr(k, true) << "];\n";
        else {
            o << ind << "        { const idx_t b_ = " << offset_expr(k, false) << ";\n";
            o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) x_" << nm << "[u].e[e_] = q_" << nm
              << "[b_ + (idx_t)e_ * p.st_" << nm << "[" << in_d << "]]; }\n";
        }
    }
    o << ind << "    }\n" << ind << "}\n";

    // phase B: evaluate, accumulate, store
    o << ind << "#pragma unroll\n" << ind << "for (int u = 0; u < " << U << "; ++u) {\n";
    o << ind << "    if (!ok[u]) continue;\n";
    for (int k : ew_out_ops) o << ind << "    ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
    o << ind << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
    EmitCtx cx;
    cx.input = [&](int k) {
        const Operand &op = c.ops[k];
        if (op.access == Access::Splat) return "ewf_in(x_" + opname(k) + "[u])";
        return "ewf_in(x_" + opname(k) + "[u].e[e_])";
    };
    cx.coord = [&](int d) {
        std::string s = "o" + std::to_string(d);
        if (T[d] > 1) s += " + c" + std::to_string(d) + "[u]";
        if (d == in_d) s += " + e_";
        return s;
    };
    emit_values(need, cx, ind + "        ");
    if (with_reduce)
        emit_accumulate("acc", level, [&](int node) { return cx.coord(argmax_canon_dim(node)); }, ind + "        ");
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
            o << ind << "    " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + (" << offset_expr(k, false) << "), y_" << nm << ");\n";
        else {
            o << ind << "    { const idx_t b_ = " << offset_expr(k, op.access == Access::Splat) << ";\n";
            o << ind << "      _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) q_" << nm << "[b_ + (idx_t)e_ * p.st_" << nm
              << "[" << in_d << "]] = y_" << nm << ".e[e_]; }\n";
        }
    }
    o << ind << "}\n";
    if (looped) { ind = ind0; o << ind << "}\n"; }

    if (with_reduce) {
        // Every wavefront folds its own lanes with cross-lane moves and stores one partial:
        // no LDS, no barrier, no atomic -- the waves of a workgroup never wait for each other
        // and the kernel streams like a copy.  A second, tiny kernel folds the partials of a
        // group in a fixed order (deterministic, and ordered by the kernel boundary alone).
        o << ind << "idx_t group = 0, slot = 0;\n";
        for (int d = 0; d < R; d++) {
            if (c.reduced[d]) o << ind << "slot = slot * p.ntile[" << d << "] + ti" << d << ";\n";
            else o << ind << "group = group * p.ext[" << d << "] + o" << d << ";\n";
        }
        o << ind << "acc = ewf_wave_reduce(acc, Acc_combine());\n";
        o << ind << "if ((tid & 63) == 0) partials[((size_t)group * (size_t)p.nslots + (size_t)slot) * EWF_NWAVES + (tid >> 6)] = acc;\n";
    }
    o << "    }\n}\n";

    if (with_reduce) {
        o << "\n// folds the partials of each reduction group, one wavefront per group\n";
        o << "extern \"C\" __global__ void __launch_bounds__(64) ewf_finish(const Params p)\n{\n";
        o << "    const int lane = threadIdx.x;\n";
        o << "    const Acc *const partials = (const Acc *)p.ws_partials;\n";
        o << "    const idx_t nparts = p.nslots * EWF_NWAVES;\n";
        o << "    for (idx_t group = blockIdx.x; group < p.nrows; group += gridDim.x) {\n";
        o << "        const Acc *const gpart = partials + (size_t)group * (size_t)nparts;\n";
        o << "        Acc tot = Acc_identity();\n";
        o << "        for (idx_t i = lane; i < nparts; i += 64) tot = Acc_combine()(tot, gpart[i]);\n";
        o << "        tot = ewf_wave_reduce(tot, Acc_combine());\n";
        o << "        if (lane != 0) continue;\n";
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
            int v = g.outputs[op.index].value;
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            emit_base(k, all_dims, "        ");
            o << "        q_" << opname(k) << "[0] = " << cv << "(v" << v << ");\n";
        }
        o << "    }\n}\n";
    }

    // ---- launch geometry and argument block
    int64_t cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : (int64_t)1 << 22;
    p.grid = std::max<int64_t>(1, std::min(ntiles, cap));
    p.lds_bytes = 0;
    int64_t ngroups = 1, nslots = 1;
    for (int d = 0; d < R; d++) { if (c.reduced[d]) nslots *= ntile[d]; else ngroups *= c.extent[d]; }
    p.counter_bytes = 0;
    p.workspace_bytes = 0;
    p.finish_grid = 0;
    if (with_reduce) {
        if (ngroups >= ((int64_t)1 << 31) || nslots >= ((int64_t)1 << 31)) return fail("too many reduction groups");
        size_t acc_bytes = 0;
        for (int n : level) acc_bytes += (g.nodes[n].op == EWF_RARGMAX) ? 8 : 4;
        p.workspace_bytes = (size_t)ngroups * (size_t)nslots * (size_t)(block / 64) * acc_bytes;
        p.finish_grid = std::min<int64_t>(ngroups, (int64_t)1 << 20);
        p.finish_block = 64;
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
    for (int n : red.level_nodes) lvl[red.edepth[n]].push_back(n);

    // which inputs vary along the row and are read by some per-element computation
    std::vector<int> elem_targets;
    for (int n : red.level_nodes) elem_targets.push_back(g.nodes[n].args[0]);
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
    const int U = resident ? (int)NV : (e.opts.unroll > 0 ? e.opts.unroll : 4);
    p.tile[in_d] = cols;

    emit_header(block);
    build_layout();
    for (int l = 1; l <= D; l++) emit_acc_struct("Acc" + std::to_string(l), lvl[l]);
    const bool has_cross = !red.cross_nodes.empty();
    if (has_cross) emit_acc_struct("AccX", red.cross_nodes);

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    o << "    const idx_t cols = p.ext[" << in_d << "];\n";
    for (int l = 1; l <= D; l++) o << "    __shared__ Acc" << l << " sm_acc" << l << "[EWF_NWAVES];\n";
    if (has_cross) o << "    AccX *const partials = (AccX *)p.ws_partials;\n";
    o << "    for (idx_t row = blockIdx.x; row < p.nrows; row += gridDim.x) {\n";
    o << "        idx_t t_ = row;\n";
    std::vector<int> outer;
    for (int d = R - 2; d >= 0; d--) {
        if (d > 0) o << "        const idx_t o" << d << " = t_ % p.ext[" << d << "]; t_ /= p.ext[" << d << "];\n";
        else o << "        const idx_t o0 = t_;\n";
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
    auto open_pass = [&](bool load) {
        if (resident) {
            o << "        #pragma unroll\n        for (int u = 0; u < " << U << "; ++u) {\n";
            o << "            const idx_t col = (idx_t)(u * EWF_BLOCK + tid) * EWF_VEC;\n";
            o << "            if (col >= cols) continue;\n";
        } else {
            o << "        for (idx_t c0 = 0; c0 < cols; c0 += " << (per_iter * U) << ") {\n";
            o << "        #pragma unroll\n        for (int u = 0; u < " << U << "; ++u) {\n";
            o << "            const idx_t col = c0 + (idx_t)(u * EWF_BLOCK + tid) * EWF_VEC;\n";
            o << "            if (col >= cols) continue;\n";
        }
        (void)load;
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

    if (resident) {
        for (int k : row_ops) o << "        ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
        open_pass(true);
        for (int k : row_ops) emit_row_load(k, "            ", "x_" + opname(k) + "[u]");
        close_pass();
    }
    for (int k : splat_ops) o << "        const " << ctype(c.ops[k].storage) << " g_" << opname(k) << " = q_" << opname(k) << "[0];\n";

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

    for (int l = 1; l <= D; l++) {
        std::string an = "Acc" + std::to_string(l), av = "acc" + std::to_string(l);
        std::vector<int> tg;
        for (int n : lvl[l]) tg.push_back(g.nodes[n].args[0]);
        std::vector<char> need = needed(tg);
        o << "        " << an << " " << av << " = " << an << "_identity();\n";
        open_pass(false);
        stream_loads(need);
        o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        emit_values(need, cx, "                ");
        emit_accumulate(av, lvl[l], [&](int node) { return cx.coord(argmax_canon_dim(node)); }, "                ");
        o << "            }\n";
        close_pass();
        o << "        " << av << " = ewf_block_reduce<EWF_NWAVES>(" << av << ", " << an << "_combine(), sm_acc" << l << ", tid);\n";
        emit_results(av, lvl[l], "        ");
    }

    if (!full_out_ops.empty()) {
        std::vector<int> tg;
        for (int k : full_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> need = needed(tg);
        open_pass(false);
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
                if (std::find(splat_ops.begin(), splat_ops.end(), k) != splat_ops.end()) continue;
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
                    const Node &nd = g.nodes[red.cross_nodes[i]];
                    o << "            ax.a" << i << " = v" << nd.args[0] << ";\n";
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
    int64_t nrows = 1;
    for (int d = 0; d < R - 1; d++) nrows *= c.extent[d];
    if (nrows >= ((int64_t)1 << 31) - 1) return fail("too many rows");
    int64_t cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : (int64_t)256 * 32;
    p.grid = std::max<int64_t>(1, std::min(nrows, cap));
    p.lds_bytes = 0;
    p.counter_bytes = 0;
    p.workspace_bytes = 0;
    p.finish_grid = 0;
    if (has_cross) {
        size_t acc_bytes = 0;
        for (int n : red.cross_nodes) acc_bytes += (g.nodes[n].op == EWF_RARGMAX) ? 8 : 4;
        p.workspace_bytes = (size_t)nrows * acc_bytes;
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

ewf_status generate(const Exec &e, Plan &p)
{
    Gen gen(e, p);
    switch (p.kclass) {
    case KernelClass::Tile: return gen.gen_tile(false);
    case KernelClass::TileReduce: return gen.gen_tile(true);
    case KernelClass::Row: return gen.gen_row();
    default: set_error("no kernel class"); return EWF_EUNSUPPORTED;
    }
}

}  // namespace ewf
