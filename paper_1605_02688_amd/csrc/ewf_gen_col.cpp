#include "ewf_gen.h"

namespace ewf {

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
    const bool small = c.total / VEC < (int64_t)256 * 512;
    // A small problem is bound by launches, not bandwidth: when one workgroup can take whole
    // columns (a single reduced dimension of modest extent) the column strips are narrowed until
    // there are enough workgroups, each folds its columns completely and writes the results
    // itself -- one launch, no workspace.
    int nreduced = 0;
    for (int d = 0; d < R; d++) nreduced += c.reduced[d];
    const bool whole_columns = small && nreduced == 1 && c.extent[dR] <= 1024 && e.opts.tile_elems <= 0;
    if (whole_columns) {
        int64_t other = 1;
        for (int d = 0; d < R - 1; d++) if (d != dR) other *= c.extent[d];
        const int min_tx = std::max(1, 16 / VEC);
        while (TX > min_tx && ceil_div(c.extent[in_d], (int64_t)TX * VEC) * other < 64) TX /= 2;
    }
    // Few columns and few rows: the lanes that neither would use take neighbouring indices of
    // the innermost other kept dimension (dK), TZ of them per workgroup, each with its own
    // columns-by-rows patch that folds inside a wavefront.  ([2097152, 4, 8] summed over axis 1:
    // two million 32-element tiles took 1.9 ms; with 32 outer indices per workgroup the tile is
    // a contiguous 4 KB.)
    int dK = -1;
    for (int d = R - 2; d >= 0; d--) if (!c.reduced[d]) { dK = d; break; }
    int TY = block / TX, TZ = 1;
    {
        // (the patch of one outer index has to fit a wavefront, inside which its row groups fold)
        // A thread takes up to four rows, but the lanes of one outer index should still read at
        // least a 128-byte line together ([2097152, 4, 8] over axis 1: 3.1 TB/s with four row lanes,
        // 1.7 TB/s with four rows per thread and 32-byte pieces; [262144, 16, 16]: 5.4 TB/s with four
        // rows per thread, 3.0 TB/s with sixteen row lanes and a quarter of the work per workgroup).
        int min_isz = 4;
        for (const Operand &op : c.ops) if (op.stride[in_d] != 0) min_isz = std::min(min_isz, isz(op.storage));
        const int rows_per_thread = e.opts.unroll > 0 ? e.opts.unroll : small ? 1 : 4;
        int ty_cap = 1;
        while (ty_cap < c.extent[dR] && ty_cap < block / TX) ty_cap *= 2;
        int ty = 1;
        while (ty < ceil_div(c.extent[dR], rows_per_thread) && ty < ty_cap) ty *= 2;
        while (ty < ty_cap && TX * ty * VEC * min_isz < 128) ty *= 2;
        if (dK >= 0 && TX * ty <= 64 && block / (TX * ty) >= 2 && c.extent[dK] >= 2 && e.opts.tile_elems <= 0) {
            TY = ty;
            TZ = block / (TX * TY);
        }
    }
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
    int U = e.opts.unroll > 0 ? e.opts.unroll : small ? 1 : heavy >= 4 ? 2 : 4;
    // (with element-wise outputs, 16 elements per thread and trip: bias + ReLU + column sums on
    // float16 [401408, 256] took 91 us with two rows of eight in flight, 119 us with four)
    if (e.opts.unroll <= 0 && !ew_out_ops.empty() && U * VEC > 16) U = std::max(1, 16 / VEC);
    // (a read-only kernel whose column count or alignment allows only narrow accesses keeps eight
    // rows in flight: float16 [1048576, 49] summed over axis 0 35 -> 25 us, [16777216, 3] 34 -> 23 us)
    {
        int narrowest = 4;
        for (const Operand &op : c.ops) if (!op.is_output && op.stride[in_d] != 0) narrowest = std::min(narrowest, isz(op.storage));
        if (e.opts.unroll <= 0 && ew_out_ops.empty() && !small && VEC * narrowest < 16) U = 8;
        // (... and one whose accesses are 16 bytes wide a single one: as for a plain copy, one wide
        // access per thread and more workgroup trips stream best.  Sums over axis 0, 268 MB: float32
        // [65536, 1024] 45.6 -> 43.0 us, [16384, 4096] 46.2 -> 42.8 us, [262144, 256] 48.4 -> 45.0 us,
        // float16 [131072, 1024] 49.5 -> 48.2 us; two in flight 43.4-46.9 us, three 46.9-55.2 us)
        else if (e.opts.unroll <= 0 && ew_out_ops.empty() && !small && TZ == 1 && heavy < 4) U = 1;
    }
    // Outer-index lanes whose rows need fewer loads than that take further outer indices, UZ in
    // all, so that a thread still has U loads in flight: with one 16-byte load per thread and
    // tile the kernel waits on memory latency (3.1 to 3.7 TB/s for [2097152, 4, 8] over axis 1).
    int UZ = 1;
    if (TZ > 1) {
        const int rpt = (int)ceil_div(c.extent[dR], TY);
        if (rpt <= U) {
            while (UZ * 2 * rpt <= U && (int64_t)UZ * TZ < c.extent[dK]) UZ *= 2;
            U = rpt;
        }
    }
    int64_t T[kMaxDims];
    for (int d = 0; d < kMaxDims; d++) T[d] = 1;
    T[in_d] = TK;
    if (TZ > 1) T[dK] = std::min<int64_t>(c.extent[dK], (int64_t)TZ * UZ);
    {
        // rows per tile: whole trips of the workgroup, and about five workgroups per CU, which all
        // run at once.  (Measured on 16 MB to 1 GB: 1280 tiles beat 4096 by 5 to 25 % -- fewer
        // partial results for the second kernel, no trailing round of workgroups -- and fewer
        // than 1024 leave CUs short of loads in flight.)
        int64_t other = ceil_div(c.extent[in_d], TK);
        for (int d = 0; d < R - 1; d++) if (d != dR) other *= c.extent[d];
        // A kernel that also streams element-wise outputs wants every CU full of wavefronts
        // instead, and short tiles: about 48 per CU (float32 [1605632, 64], bias + ReLU + column
        // sums: 12544 tiles 146 us, 1255 tiles 165 us, 100352 tiles 194 us).
        const int64_t want = (int64_t)(ew_out_ops.empty() ? 5 : 48) * device_cu_count();
        const int64_t trip = (int64_t)TY * U;
        // (at least 128 bytes of every column per tile, or the partial results, one 4-byte value
        // per column and tile, become a noticeable part of the traffic)
        int in_sz = 4;
        for (const Operand &op : c.ops) if (!op.is_output && op.stride[in_d] != 0) in_sz = std::min(in_sz, isz(op.storage));
        const int64_t min_rows = std::max<int64_t>(trip, 128 / in_sz);
        int64_t slices = std::max<int64_t>(1, std::min(ceil_div(want, other), ceil_div(c.extent[dR], min_rows)));
        if (whole_columns || TZ > 1) slices = 1;
        int64_t tr = ceil_div(c.extent[dR], slices);
        if (slices > 1) tr = std::max(trip, (tr + trip / 2) / trip * trip);
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

    const bool one_tile = nslots == 1;
    const int NW = block / 64;
    // The second kernel folds a column's partial results either with the lanes of a workgroup
    // (many slots) or in one thread per column (few slots, or a moderate number under so many
    // columns that the threads fill the chip anyway: 65536 columns of 32 slots took 28 us with a
    // 64-lane workgroup each).
    const bool fin_lanes = nslots > 16 && !(nslots <= 128 && ngroups >= 64 * nslots);
    const int fin_block = nslots > 256 ? 256 : 64;

    // ---- what to evaluate per element
    std::vector<int> targets;
    for (int k : ew_out_ops) targets.push_back(g.outputs[c.ops[k].index].value);
    for (int n : level) targets.push_back(g.nodes[n].args[0]);
    std::vector<char> need = needed(targets);
    std::vector<int> load_ops = inputs_of(need);

    emit_header(block);
    o << "#define EWF_TX " << TX << "\n#define EWF_TY " << TY << "\n#define EWF_TZ " << TZ << "\n";
    build_layout();
    emit_acc_struct("Acc", level);
    std::vector<int> all_dims;
    for (int d = 0; d < R; d++) all_dims.push_back(d);

    const std::string tzs = UZ > 1 ? "tzz_" : "tz";          // the thread's outer index inside the tile
    const std::string okname = UZ > 1 ? "zok_" : "colok_";   // its columns (and outer index) exist
    std::string xi = "u";                                    // where a row's loaded values are kept
    auto off_expr = [&](int k) {
        // offset of (row r_, column cc_) from the tile's origin
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        std::string s;
        if (op.stride[dR] != 0) s = "(ioff_t)r_ * (ioff_t)p.st_" + nm + "[" + std::to_string(dR) + "]";
        if (TZ > 1 && op.stride[dK] != 0) {
            if (!s.empty()) s += " + ";
            s += "(ioff_t)" + tzs + " * (ioff_t)p.st_" + nm + "[" + std::to_string(dK) + "]";
        }
        if (op.stride[in_d] != 0) {
            if (!s.empty()) s += " + ";
            s += op.stride[in_d] == 1 ? std::string("(ioff_t)cc_") : "(ioff_t)cc_ * (ioff_t)p.st_" + nm + "[" + std::to_string(in_d) + "]";
        }
        return s.empty() ? std::string("(ioff_t)0") : s;
    };

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    o << "    const int tx = tid & (EWF_TX - 1), ty = (tid / EWF_TX) & (EWF_TY - 1), tz = tid / (EWF_TX * EWF_TY);\n";
    o << "    (void)tz;\n";
    if (!one_tile) o << "    Acc *const partials = (Acc *)p.ws_partials;\n";
    if (NW > 1 && TZ == 1) o << "    __shared__ Acc sm_col[(EWF_NWAVES - 1) * EWF_TX * EWF_VEC];\n";
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
    o << ind << "const bool colok_ = cc_ < " << TK << " && o" << in_d << " + cc_ < p.ext[" << in_d << "]"
      << (TZ > 1 && UZ == 1 ? " && o" + std::to_string(dK) + " + tz < p.ext[" + std::to_string(dK) + "]" : std::string("")) << ";\n";
    o << ind << "const int rows_ = (int)((p.ext[" << dR << "] - o" << dR << ") < " << TR << " ? (p.ext[" << dR << "] - o" << dR << ") : " << TR << ");\n";
    // An operand that is the same for every row of the tile (a per-column bias) is loaded once
    // per tile, not once per row: fewer load instructions and U times fewer registers.
    auto tile_invariant = [&](int k) {
        const Operand &op = c.ops[k];
        return op.stride[dR] == 0 && (TZ == 1 || op.stride[dK] == 0);
    };
    EmitCtx cx;
    cx.input = [&](int k) {
        const Operand &op = c.ops[k];
        const std::string at = tile_invariant(k) ? std::string("") : "[" + xi + "]";
        if (op.stride[in_d] == 0) return "ewf_in(x_" + opname(k) + at + ")";
        if (op.storage == EWF_F16 && VEC >= 2) return "ewf_in_h(x_" + opname(k) + at + ", e_)";
        return "ewf_in(x_" + opname(k) + at + ".e[e_])";
    };
    auto emit_load = [&](int k, const std::string &at, const std::string &in2) {
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        if (op.stride[in_d] == 0)
            o << in2 << "x_" << nm << at << " = *ewf_at(q_" << nm << ", " << off_expr(k) << ");\n";
        else if (op.access == Access::Vector)
            o << in2 << "x_" << nm << at << " = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << off_expr(k) << "));\n";
        else {
            o << in2 << "{ const ioff_t b_ = " << off_expr(k) << ";\n";
            o << in2 << "  _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) x_" << nm << at << ".e[e_] = *ewf_at(q_" << nm
              << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm << "[" << in_d << "]); }\n";
        }
    };
    for (int k : load_ops) {
        if (!tile_invariant(k)) continue;
        const Operand &op = c.ops[k];
        if (op.stride[in_d] == 0) o << ind << ctype(op.storage) << " x_" << opname(k) << ";\n";
        else o << ind << "ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << ";\n";
        o << ind << "if (colok_) {\n";
        emit_load(k, "", ind + "    ");
        o << ind << "}\n";
    }
    cx.coord = [&](int d) {
        std::string s = "o" + std::to_string(d);
        if (d == dR) s += " + r_";
        if (TZ > 1 && d == dK) s += " + " + tzs;
        if (d == in_d) s += " + cc_ + e_";
        return s;
    };
    auto emit_x_arrays = [&](const std::string &in2, int n) {
        for (int k : load_ops) {
            const Operand &op = c.ops[k];
            if (tile_invariant(k)) continue;
            if (op.stride[in_d] == 0) o << in2 << ctype(op.storage) << " x_" << opname(k) << "[" << n << "];\n";
            else o << in2 << "ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << "[" << n << "];\n";
        }
    };
    // the loads of the U rows of one trip (first row r0), kept at index xi
    // (guard: 0 every row of the trip exists and the lane is in range -- no branch between the
    // loads, which then go out back to back; 1 check the row; 2 check the row and the lane)
    auto emit_guard = [&](const std::string &in2, int guard) {
        if (guard == 1) o << in2 << "    if (r_ >= rows_) continue;\n";
        if (guard == 2) o << in2 << "    if (!" << okname << " || r_ >= rows_) continue;\n";
    };
    auto emit_loads = [&](const std::string &in2, const std::string &r0, int guard) {
        o << in2 << "#pragma unroll\n" << in2 << "for (int u = 0; u < " << U << "; ++u) {\n";
        o << in2 << "    const int r_ = " << r0 << " + u * EWF_TY;\n";
        emit_guard(in2, guard);
        for (int k : load_ops) if (!tile_invariant(k)) emit_load(k, "[" + xi + "]", in2 + "    ");
        o << in2 << "}\n";
    };
    // their arithmetic, accumulation and element-wise stores
    auto emit_arith = [&](const std::string &in2, const std::string &r0, int guard) {
        o << in2 << "#pragma unroll\n" << in2 << "for (int u = 0; u < " << U << "; ++u) {\n";
        o << in2 << "    const int r_ = " << r0 << " + u * EWF_TY;\n";
        emit_guard(in2, guard);
        for (int k : ew_out_ops) o << in2 << "    ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
        o << in2 << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        emit_values(need, cx, in2 + "        ");
        emit_accumulate("acc[e_]", level, [&](int node) { return argmax_index(node, cx.coord); }, in2 + "        ");
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << in2 << "        y_" << opname(k) << ".e[e_] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
        }
        o << in2 << "    }\n";
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            const std::string nm = opname(k);
            if (op.access == Access::Vector)
                o << in2 << "    " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << off_expr(k) << "), y_" << nm << ");\n";
            else {
                o << in2 << "    { const ioff_t b_ = " << off_expr(k) << ";\n";
                o << in2 << "      _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) *ewf_at(q_" << nm << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm
                  << "[" << in_d << "]) = y_" << nm << ".e[e_]; }\n";
            }
        }
        o << in2 << "}\n";
    };
    // The row groups inside a wavefront (lanes that differ by a multiple of TX) fold with lane
    // exchanges in a fixed butterfly; the wavefronts then meet in LDS and the first folds them
    // in order.  Then the tile's partial results (or, with one tile per column, the results) go out.
    auto emit_fold_and_write = [&](const std::string &in2) {
        for (int m = TX; m < (TZ > 1 ? TX * TY : 64); m *= 2)
            o << in2 << "_Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) acc[e_] = Acc_combine()(acc[e_], ewf_lane_xor(acc[e_], " << m << "));\n";
        if (NW > 1 && TZ == 1) {
            o << in2 << "if (tid >= 64 && (tid & 63) < EWF_TX) { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) sm_col[(((tid >> 6) - 1) * EWF_TX + tx) * EWF_VEC + e_] = acc[e_]; }\n";
            o << in2 << "__syncthreads();\n";
            o << in2 << "if (tid < EWF_TX) {\n";
            o << in2 << "    for (int w_ = 0; w_ < EWF_NWAVES - 1; ++w_)\n";
            o << in2 << "        _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) acc[e_] = Acc_combine()(acc[e_], sm_col[(w_ * EWF_TX + tx) * EWF_VEC + e_]);\n";
            o << in2 << "}\n";
        }
        o << in2 << "if (" << (TZ > 1 ? "ty == 0" : "tid < EWF_TX") << " && " << okname << ") {\n";
        o << in2 << "    size_t group = 0, slot = 0;\n";
        for (int d = 0; d < R; d++) {
            if (c.reduced[d]) o << in2 << "    slot = slot * (size_t)p.ntile[" << d << "] + (size_t)ti" << d << ";\n";
            else if (d == in_d) o << in2 << "    group = group * (size_t)p.ext[" << d << "] + (size_t)(o" << d << " + cc_);\n";
            else if (TZ > 1 && d == dK) o << in2 << "    group = group * (size_t)p.ext[" << d << "] + (size_t)(o" << d << " + " << tzs << ");\n";
            else o << in2 << "    group = group * (size_t)p.ext[" << d << "] + (size_t)o" << d << ";\n";
        }
        if (one_tile) {
            // every column is complete here: its results are written straight away, from the
            // coordinates at hand, a vector of columns per store where the output allows it
            // (element by element, the 4-byte stores of [2097152, 2, 16] summed over axis 1 took
            // longer than reading the input)
            o << in2 << "    (void)slot; (void)group;\n";
            std::vector<std::string> coords(R);
            for (int d = 0; d < R; d++) coords[d] = "gc" + std::to_string(d) + "_";
            auto vector_out = [&](int k) { return VEC > 1 && c.ops[k].access == Access::Vector && c.ops[k].stride[in_d] == 1; };
            for (int k : group_out_ops)
                if (vector_out(k))
                    o << in2 << "    ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> yg_" << opname(k) << "; "
                      << ctype(c.ops[k].storage) << " *qg_" << opname(k) << " = nullptr;\n";
            o << in2 << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
            o << in2 << "        const Acc tot = acc[e_];\n";
            for (int d = 0; d < R; d++) {
                if (c.reduced[d]) continue;
                o << in2 << "        const idx_t gc" << d << "_ = o" << d;
                if (d == in_d) o << " + cc_ + e_";
                else if (TZ > 1 && d == dK) o << " + " << tzs;
                o << ";\n";
            }
            const GroupStore store = [&](int k, const std::string &value, const std::string &in3) {
                const std::string nm = opname(k);
                if (vector_out(k)) o << in3 << "if (e_ == 0) qg_" << nm << " = q_" << nm << ";\n" << in3 << "yg_" << nm << ".e[e_] = " << value << ";\n";
                else o << in3 << "q_" << nm << "[0] = " << value << ";\n";
            };
            o << in2 << "        {\n";
            emit_group_epilogue(level, group_out_ops, std::vector<Gather>(), in2 + "            ", &coords, &store);
            o << in2 << "        }\n";
            o << in2 << "    }\n";
            for (int k : group_out_ops)
                if (vector_out(k))
                    o << in2 << "    " << (c.ops[k].stream ? "ewf_st_nt<" : "ewf_st<") << ctype(c.ops[k].storage) << ", EWF_VEC>(qg_" << opname(k) << ", yg_" << opname(k) << ");\n";
        }
        else if (fin_lanes) o << in2 << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) partials[(group + e_) * (size_t)p.nslots + slot] = acc[e_];\n";
        else o << in2 << "    _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) partials[slot * (size_t)p.nrows + group + e_] = acc[e_];\n";
        o << in2 << "}\n";
        if (NW > 1 && TZ == 1) o << in2 << "__syncthreads();\n";
    };
    const std::string acc_init = "_Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) acc[e_] = Acc_identity();\n";
    if (UZ == 1) {
        o << ind << "Acc acc[EWF_VEC];\n" << ind << acc_init;
        // whole trips without a branch, then at most one trip that checks its rows (with the
        // checks between them the loads waited for one another: bias + ReLU + column sums on
        // float32 [401408, 256] ran at 5.2 TB/s)
        o << ind << "if (colok_) {\n";
        o << ind << "    int r0_ = ty;\n";
        o << ind << "    for (; r0_ + " << (U - 1) << " * EWF_TY < rows_; r0_ += EWF_TY * " << U << ") {\n";
        emit_x_arrays(ind + "        ", U);
        emit_loads(ind + "        ", "r0_", 0);
        emit_arith(ind + "        ", "r0_", 0);
        o << ind << "    }\n";
        if (U > 1) {
            o << ind << "    if (r0_ < rows_) {\n";
            emit_x_arrays(ind + "        ", U);
            emit_loads(ind + "        ", "r0_", 1);
            emit_arith(ind + "        ", "r0_", 1);
            o << ind << "    }\n";
        }
        o << ind << "}\n";
        emit_fold_and_write(ind);
    }
    else {
        // all the rows of a patch fit one trip: the loads of the thread's UZ outer indices go out
        // together, then each index is folded and written in turn
        const std::string zhead = "    const int tzz_ = tz + z_ * EWF_TZ;\n" + ind +
            "    const bool zok_ = colok_ && o" + std::to_string(dK) + " + tzz_ < p.ext[" + std::to_string(dK) + "];\n";
        xi = "z_ * " + std::to_string(U) + " + u";
        emit_x_arrays(ind, UZ * U);
        // (a thread whose outer indices and rows all exist issues its loads without a branch)
        o << ind << "const bool all_ = colok_ && o" << dK << " + tz + " << (UZ - 1) << " * EWF_TZ < p.ext[" << dK << "] && ty + "
          << (U - 1) << " * EWF_TY < rows_;\n";
        for (int guard : {0, 2}) {
            o << ind << (guard == 0 ? "if (all_) {\n" : "else {\n");
            o << ind << "    #pragma unroll\n" << ind << "    for (int z_ = 0; z_ < " << UZ << "; ++z_) {\n" << ind << "    " << zhead;
            o << ind << "        (void)zok_;\n";
            emit_loads(ind + "        ", "ty", guard);
            o << ind << "    }\n" << ind << "}\n";
        }
        o << ind << "#pragma unroll\n" << ind << "for (int z_ = 0; z_ < " << UZ << "; ++z_) {\n" << ind << zhead;
        o << ind << "    Acc acc[EWF_VEC];\n" << ind << "    " << acc_init;
        emit_arith(ind + "    ", "ty", 2);
        emit_fold_and_write(ind + "    ");
        o << ind << "}\n";
    }
    o << "    }\n}\n";

    // ---- second kernel.  Many slots per column: the partials of a column are contiguous and a
    // workgroup's lanes walk them.  Few: one thread per column folds its slots in slot order.
    if (one_tile) { /* no second kernel */ }
    else if (fin_lanes) emit_finish_lanes(level, group_out_ops, "p.nslots", fin_block,
                                     (int)std::min<int64_t>(8, std::max<int64_t>(1, ceil_div(nslots, fin_block))));
    else {
    o << "\nextern \"C\" __global__ void __launch_bounds__(256) ewf_finish(const Params p)\n{\n";
    o << "    const Acc *const partials = (const Acc *)p.ws_partials;\n";
    o << "    for (idx_t group = blockIdx.x * 256 + threadIdx.x; group < p.nrows; group += gridDim.x * 256) {\n";
    o << "        Acc tot = partials[group];\n";
    o << "        _Pragma(\"unroll 8\") for (idx_t s_ = 1; s_ < p.nslots; ++s_) tot = Acc_combine()(tot, partials[(size_t)s_ * (size_t)p.nrows + (size_t)group]);\n";
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
    // With outer-index lanes a tile is a few KB, too little to pay for a workgroup's start: a
    // resident grid that walks the tiles is 10 to 25 % faster there (and slower everywhere else).
    int64_t cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : TZ > 1 ? (int64_t)16 * device_cu_count() : (int64_t)1 << 22;
    p.grid = std::max<int64_t>(1, std::min(ntiles, cap));
    p.lds_bytes = NW > 1 && TZ == 1 ? (int)((NW - 1) * TX * VEC * acc_bytes(level)) : 0;
    if (p.lds_bytes > 60 * 1024) return fail("too many reductions for one column kernel (LDS)");
    p.staged = 0;
    p.workspace_bytes = one_tile ? 0 : (size_t)ngroups * (size_t)nslots * acc_bytes(level);
    p.finish_grid = one_tile ? 0 : fin_lanes ? std::min<int64_t>(ngroups, (int64_t)1 << 20)
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


}  // namespace ewf
