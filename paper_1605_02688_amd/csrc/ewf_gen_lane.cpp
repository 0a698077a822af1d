#include "ewf_gen.h"

namespace ewf {

// =========================================================================================
// Lane: short rows, several rows per wavefront
//
// When the innermost (reduced) dimension is short, a wavefront per row leaves most lanes idle
// (rows of 8 floats: 2 lanes of 64 at work).  Here a group of L lanes owns a row, L a power of
// two from 1 (a row of up to 32 bytes: one thread loads it whole) to 64: every lane loads its
// vectors of the row into registers, the chained reduction levels run over them, the L lanes of
// a row fold with a butterfly of lane exchanges (none when L is 1) after which each of them
// holds the row's result, and every lane writes the element-wise outputs of its own columns.
// Neighbouring lane groups hold neighbouring rows, so a wavefront reads one contiguous piece of
// memory.  The row length is a compile-time constant of the generated text (it is part of the
// plan's key).

ewf_status Gen::gen_lane()
{
    const int in_d = R - 1;
    const int64_t cols = c.extent[in_d];
    const int block = e.opts.block_threads > 0 ? e.opts.block_threads : 256;
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");
    p.block = block;
    const int nin = g.ninputs;
    if (cols % VEC) return fail("row length is not a multiple of the vector width");
    // lanes per row, vectors per lane
    int min_isz = 4;
    for (const Operand &op : c.ops) if (op.stride[in_d] != 0) min_isz = std::min(min_isz, isz(op.storage));
    int L = 1;
    const int64_t nvec = cols / VEC;
    if (cols * min_isz > 32) while (L < 64 && L < nvec) L *= 2;
    // more vectors than lanes (narrow vectors: an odd row length, or rows that are not aligned):
    // the lane count that leaves the fewest lane slots idle, with at most 16 vectors per lane
    // (rows of 130 float32 are 65 pairs: 64 lanes would take two trips with 63 idle slots, 8 lanes
    // take nine with 7)
    // (... and at most 64 registers of row data per lane: two float32 operands with rows of 784
    // are held by 32 lanes, seven vectors of each, not by 16 lanes with thirteen)
    if (nvec > 64) {
        int vec_regs = 0;                               // registers that one vector of every row operand takes
        for (int k = 0; k < nin; k++)
            if (c.ops[k].stride[in_d] != 0 && live[g.input_node[k]]) vec_regs += (VEC * isz(c.ops[k].storage) + 3) / 4;
        int64_t best_waste = -1;
        for (int l = 64; l >= 8; l /= 2) {
            const int64_t nv = ceil_div(nvec, (int64_t)l), waste = nv * l - nvec;
            if (nv > 16 || (l < 64 && nv * vec_regs > 64)) break;
            if (best_waste < 0 || waste < best_waste) { best_waste = waste; L = l; }
        }
    }
    // ... but at least 16 bytes of the row per lane: where the row length or the alignment allows
    // only narrow accesses, a lane with a single one in flight leaves the memory system idle
    // (rows of 49 float32, one element per lane: 2.9 TB/s)
    while (L > 1 && ceil_div(cols, (int64_t)L * VEC) * VEC * min_isz < 16) L /= 2;
    // (two lanes that interleave narrow pieces of a short row do worse than one thread that
    // takes it whole: rows of 9 float32 4.4 against 6 TB/s, rows of 25 float16 2.9 against 6)
    if (L == 2 && VEC * min_isz < 16 && cols / VEC <= 32) L = 1;
    const int64_t NV = ceil_div(cols, (int64_t)L * VEC);
    const bool ragged_cols = NV * L * VEC != cols;

    // ---- roles of the outputs
    std::vector<int> full_out_ops, group_out_ops, final_out_ops;
    for (size_t k = nin; k < c.ops.size(); k++) {
        int vn = g.outputs[c.ops[k].index].value;
        const Node &v = g.nodes[vn];
        if (after_cross[vn]) final_out_ops.push_back((int)k);
        else if ((v.bcast & red.axes) == red.axes) group_out_ops.push_back((int)k);
        else full_out_ops.push_back((int)k);
    }
    const int D = red.max_depth;
    std::vector<std::vector<int>> lvl(D + 1);
    std::vector<std::vector<Gather>> gat(D + 1);
    for (int n : red.level_nodes) {
        Gather ga;
        if (match_gather(n, ga) && ga.cdim == in_d) gat[red.edepth[n]].push_back(ga);
        else lvl[red.edepth[n]].push_back(n);
    }
    std::vector<int> elem_targets;
    for (int l = 1; l <= D; l++) for (int n : lvl[l]) elem_targets.push_back(g.nodes[n].args[0]);
    for (int k : full_out_ops) elem_targets.push_back(g.outputs[c.ops[k].index].value);
    std::vector<char> eneed = needed(elem_targets);
    std::vector<int> row_ops, splat_ops;
    for (int k : inputs_of(eneed)) (c.ops[k].stride[in_d] != 0 ? row_ops : splat_ops).push_back(k);
    int regs = 0;
    for (int k : row_ops) regs += (int)(NV * VEC * isz(c.ops[k].storage) + 3) / 4;
    if (NV > 32 || regs > 96) return fail("a row does not fit the registers of one thread");

    int64_t nrows = 1;
    for (int d = 0; d < R - 1; d++) nrows *= c.extent[d];
    if (nrows >= ((int64_t)1 << 31) - 1) return fail("too many rows");
    p.tile[in_d] = cols;

    emit_header(block);
    build_layout();
    for (int l = 1; l <= D; l++) if (!lvl[l].empty()) emit_acc_struct("Acc" + std::to_string(l), lvl[l]);
    const bool has_cross = !red.cross_nodes.empty();
    if (has_cross) emit_acc_struct("AccX", red.cross_nodes);

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    if (has_cross) o << "    AccX *const partials = (AccX *)p.ws_partials;\n";
    // every lane of a wavefront makes the same number of trips (the lane exchanges need them all);
    // lanes past the last row work on a copy of it and store nothing
    o << "    const int lr = threadIdx.x & " << (L - 1) << ";\n";
    o << "    for (idx_t base_ = (idx_t)blockIdx.x * " << block / L << "; base_ < p.nrows; base_ += (idx_t)gridDim.x * " << block / L << ") {\n";
    o << "        const idx_t row_ = base_ + (idx_t)(threadIdx.x / " << L << ");\n";
    o << "        const bool live_ = row_ < p.nrows;\n";
    o << "        const idx_t row = live_ ? row_ : p.nrows - 1;\n";
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

    // values constant along the row: one element per thread
    std::vector<int> const_loaded = splat_ops;
    for (int l = 1; l <= D; l++)
        for (const Gather &ga : gat[l])
            for (int k : inputs_of(needed(std::vector<int>{ga.index_value})))
                if (std::find(const_loaded.begin(), const_loaded.end(), k) == const_loaded.end()) const_loaded.push_back(k);
    for (int k : const_loaded) {
        base_once(k, "        ");
        o << "        const " << ctype(c.ops[k].storage) << " g_" << opname(k) << " = q_" << opname(k) << "[0];\n";
    }
    // the row itself
    for (int k : row_ops) {
        const Operand &op = c.ops[k];
        const std::string nm = opname(k);
        o << "        ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << nm << "[" << NV << "];\n";
        o << "        #pragma unroll\n        for (int j = 0; j < " << NV << "; ++j) {\n";
        o << "            const int col = (j * " << L << " + lr) * EWF_VEC;\n";
        if (ragged_cols) o << "            if (col >= " << cols << ") continue;\n";
        if (op.access == Access::Vector)
            // (ordinary loads even for operands touched once: with one thread per row the vectors of
            // a row are separate instructions that share cache lines -- rows of 8 floats 26.3 us with
            // non-temporal loads, 22.5 us without; 32 columns 50.7 against 45.3 us)
            o << "            x_" << nm << "[j] = ewf_ld<" << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col);\n";
        else
            o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) x_" << nm << "[j].e[e_] = q_" << nm
              << "[(idx_t)(col + e_) * p.st_" << nm << "[" << in_d << "]];\n";
        o << "        }\n";
    }

    EmitCtx cx;
    cx.input = [&](int k) {
        if (c.ops[k].stride[in_d] == 0) return "ewf_in(g_" + opname(k) + ")";
        return "ewf_in(x_" + opname(k) + "[j].e[e_])";
    };
    cx.coord = [&](int d) {
        if (d == in_d) return std::string("(col + e_)");
        return "o" + std::to_string(d);
    };
    EmitCtx ux;                                         // values constant along the row
    ux.input = [&](int k) { return "ewf_in(g_" + opname(k) + ")"; };
    ux.coord = [&](int d) { return d == in_d ? std::string("0") : "o" + std::to_string(d); };

    for (int l = 1; l <= D; l++) {
        for (const Gather &ga : gat[l]) {
            std::vector<char> need = needed(std::vector<int>{ga.index_value});
            base_once(ga.input, "        ");
            const std::string nm = opname(ga.input);
            o << "        float r" << ga.node << ";\n        {\n";
            emit_values(need, ux, "            ");
            o << "            const int t_ = v" << ga.index_value << ";\n";
            o << "            const bool in_ = t_ >= 0 && t_ < " << cols << ";\n";
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
        o << "        #pragma unroll\n        for (int j = 0; j < " << NV << "; ++j) {\n";
        o << "            const int col = (j * " << L << " + lr) * EWF_VEC;\n";
        if (ragged_cols) o << "            if (col >= " << cols << ") continue;\n";
        o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
        emit_values(need, cx, "                ");
        // a lane walks its columns in increasing order
        emit_accumulate(av, lvl[l], [&](int node) { return argmax_index(node, cx.coord); }, "                ", true);
        o << "            }\n        }\n";
        emit_first_index(av, lvl[l], "lr * EWF_VEC < " + std::to_string(cols), "lr * EWF_VEC", "        ");
        // the lanes of a row fold with a fixed butterfly; afterwards each holds the row's result
        for (int m = 1; m < L; m *= 2)
            o << "        " << av << " = " << an << "_combine()(" << av << ", ewf_lane_xor(" << av << ", " << m << "));\n";
        emit_results(av, lvl[l], "        ");
    }

    if (!full_out_ops.empty()) {
        std::vector<int> tg;
        for (int k : full_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        std::vector<char> need = needed(tg);
        o << "        #pragma unroll\n        for (int j = 0; j < " << NV << "; ++j) {\n";
        o << "            const int col = (j * " << L << " + lr) * EWF_VEC;\n";
        o << "            if (!live_" << (ragged_cols ? " || col >= " + std::to_string(cols) : std::string("")) << ") continue;\n";
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
                o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) q_" << nm << "[(idx_t)(col + e_) * p.st_" << nm
                  << "[" << in_d << "]] = y_" << nm << ".e[e_];\n";
        }
        o << "        }\n";
    }

    // per-row values: results of the reductions, the outputs derived from them, and the
    // arguments of cross-row reductions -- every thread for its own row
    {
        std::vector<int> tg;
        for (int k : group_out_ops) tg.push_back(g.outputs[c.ops[k].index].value);
        for (int n : red.cross_nodes) tg.push_back(g.nodes[n].args[0]);
        if (!tg.empty()) {
            std::vector<char> need = needed(tg);
            o << "        if (live_ && lr == 0) {\n";
            for (int k : inputs_of(need)) {
                if (std::find(const_loaded.begin(), const_loaded.end(), k) != const_loaded.end()) continue;
                base_once(k, "            ");
                o << "            const " << ctype(c.ops[k].storage) << " g_" << opname(k) << " = q_" << opname(k) << "[0];\n";
            }
            emit_values(need, ux, "            ");
            for (int k : group_out_ops) {
                const Operand &op = c.ops[k];
                const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
                emit_base(k, outer, "            ");
                o << "            q_" << opname(k) << "[0] = " << cv << "(v" << g.outputs[op.index].value << ");\n";
            }
            if (has_cross) emit_cross_partial("            ");
            o << "        }\n";
        }
    }
    o << "    }\n}\n";
    int cross_block = 256;
    if (has_cross) cross_block = emit_cross_finish(final_out_ops, nrows);

    // ---- launch geometry and argument block
    // With several lanes per row a resident grid that strides over the rows streams better than
    // one short-lived workgroup per 256 / L rows (32 columns: 40.7 against 50.7 us; 128: 40.0
    // against 49.2 us); with a thread per row the short-lived workgroups win (26.3 against 30.2 us).
    const int64_t grid_cap = e.opts.max_blocks > 0 ? e.opts.max_blocks : L > 1 ? (int64_t)8 * device_cu_count() : (int64_t)1 << 20;
    p.grid = std::max<int64_t>(1, std::min(ceil_div(nrows, block / L), grid_cap));
    p.lds_bytes = 0;
    p.staged = 0;
    p.workspace_bytes = 0;
    p.finish_grid = 0;
    if (has_cross) {
        p.workspace_bytes = (size_t)nrows * acc_bytes(red.cross_nodes);
        p.finish_grid = 1;
        p.finish_block = cross_block;
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

}  // namespace ewf
