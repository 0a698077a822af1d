#include "ewf_gen.h"

namespace ewf {

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
        // at most twelve vectors of the row per thread, or 24 single elements (rows of 10001
        // float32, whose odd pitch allows no wider access: 512 threads 14.6 us, 1024 threads 22.3 us)
        while (block < 1024 && cols > (int64_t)block * std::max(VEC * 12, 24)) block *= 2;
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

    // Operands that only the element-wise outputs use (the scale and shift rows of a layer
    // normalisation) are read where those outputs are written, not held under the reductions.
    std::vector<char> late(c.ops.size(), 0);
    {
        std::vector<int> level_targets;
        for (int l = 1; l <= D; l++) for (int n : lvl[l]) level_targets.push_back(g.nodes[n].args[0]);
        std::vector<char> lneed = needed(level_targets);
        std::vector<int> under = inputs_of(lneed);
        for (int k : row_ops) if (std::find(under.begin(), under.end(), k) == under.end()) late[k] = 1;
    }
    // With such operands the last pass issues loads of its own next to the arithmetic, and more
    // threads with fewer vectors each hide them better: two vectors of the row per thread (layer
    // normalisation with scale and shift rows, 134 MB: float16 [4096, 16384] 256 threads 67.2 us,
    // 1024 threads 55.5 us; [8192, 8192] 256 threads 59.5 us, 512 threads 54.4 us; float32
    // [8192, 8192] 99.4 -> 93.0 us, [4096, 16384] 99.3 -> 91.1 us; softmax, which has none, runs
    // best as it is).
    if (e.opts.block_threads <= 0 && std::find(late.begin(), late.end(), (char)1) != late.end()) {
        int want = 64;
        while (want < 1024 && (int64_t)want * VEC * 2 < cols) want *= 2;
        if (want > block) { block = want; p.block = block; }
    }
    // ---- residency: keep the row in registers when it fits
    const int64_t per_iter = (int64_t)block * VEC;
    const int64_t NV = ceil_div(cols, per_iter);
    int regs = 0;
    for (int k : row_ops) if (!late[k]) regs += (int)NV * VEC * isz(c.ops[k].storage) / 4;
    const bool resident = NV <= 32 && regs <= 96;
    if (p.avoid_poor_rows && e.opts.split_rows != 2) {
        int64_t nr = 1;
        for (int d = 0; d < R - 1; d++) nr *= c.extent[d];
        // measured on [rows, cols] float32 softmax cross-entropy of 268 MB: rows held in registers
        // run at 5.3-5.5 TB/s up to 32768 columns but 4.1 TB/s at 65536 (64 registers per thread,
        // 1024 threads: one workgroup per compute unit), rows streamed once per level 2.7-3.4 TB/s;
        // split over workgroups 5.0-5.2 TB/s at any row length
        // (a chain that a plan in passes cannot shorten -- layer normalisation of float32
        // [4096, 16384] with its scale and shift rows: 96 registers of row data, 91 us here against
        // 185 us in three passes -- keeps the row class as long as the row fits at all)
        // (without outputs that vary along the row, from 32 registers of 1024 threads on: softmax cross-entropy on
        // float32 [1280, 32768] 40.0 us with 1024 threads a row -- two workgroups per compute unit,
        // two and a half rounds of them -- against 35.6 us split; [3000, 32768] 84.1 against 78.1 us,
        // [1280, 49152] 54.6 against 49.9 us, [20000, 32768] 450 against 411 us; [512, 40000] 22.1 against 23.3 us)
        const bool too_long = !resident || (regs > 48 && p.fused_depth <= 1) ||
                              (block == 1024 && regs >= 32 && p.fused_depth <= 1 && full_out_ops.empty());
        if (too_long || (nr * 2 < device_cu_count() && cols >= 16384) || e.opts.split_rows == 1) {
            p.row_refused = true;
            return fail(too_long ? "a row does not fit the registers of a workgroup well: the row class would read it once per reduction level or run one workgroup per compute unit"
                                 : "too few rows for one workgroup per row to occupy the chip");
        }
    }
    const int U = resident ? (int)NV : (e.opts.unroll > 0 ? e.opts.unroll : 4);
    p.tile[in_d] = cols;
    // Maxima and arg-maxima of a float input row that waits in registers are taken the cheap way
    // first: the hardware maximum (which drops NaN) next to a check word that turns NaN when the
    // row holds a NaN or an infinity, then the index by the threads that hold the maximum.  Only a
    // row whose check word is NaN is folded again with the rules that rank NaN.  (Per element: one
    // and a half instructions instead of five on a dependent chain.)
    std::vector<std::vector<int>> fastn(D + 1);
    std::vector<int> fast_op(D + 1, -1);
    if (resident && !e.opts.plain_extremes) {
        for (int l = 1; l <= D; l++) {
            int arg = -1;
            std::vector<int> rest;
            for (int n : lvl[l]) {
                const Node &nd = g.nodes[n];
                const Node &a = g.nodes[nd.args[0]];
                bool take = (nd.op == EWF_RMAX || nd.op == EWF_RARGMAX) && a.vtype == EWF_F32 && a.kind == NodeKind::Input &&
                            std::find(row_ops.begin(), row_ops.end(), a.index) != row_ops.end() && !late[a.index] &&
                            (arg < 0 || arg == nd.args[0]);
                if (take) { arg = nd.args[0]; fastn[l].push_back(n); fast_op[l] = a.index; }
                else rest.push_back(n);
            }
            lvl[l] = rest;
        }
    }
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
    for (int l = 1; l <= D; l++) if (!fastn[l].empty()) emit_acc_struct("AccS" + std::to_string(l), fastn[l]);
    const bool has_cross = !red.cross_nodes.empty();
    if (has_cross) emit_acc_struct("AccX", red.cross_nodes);

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    o << "    const idx_t cols = p.ext[" << in_d << "];\n";
    for (int l = 1; l <= D; l++) if (!lvl[l].empty()) o << "    __shared__ Acc" << l << " sm_acc" << l << "[EWF_NWAVES];\n";
    for (int l = 1; l <= D; l++)
        if (!fastn[l].empty())
            o << "    __shared__ AccS" << l << " sm_accs" << l << "[EWF_NWAVES];\n    __shared__ ewf_fmax sm_fm" << l
              << "[EWF_NWAVES];\n    __shared__ int sm_ix" << l << "[EWF_NWAVES];\n";
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
    // Vectors that assume element alignment only (see Plan::loose_vec): a row may start at any
    // element, and when its length is no whole number of vectors the last one is cut (`ragged`)
    // and handled element by element.  The steps below NFULL hold whole vectors for every thread,
    // which the unrolled code knows at compile time.
    const bool loose = p.loose_vec;
    const bool ragged = loose && cols % VEC != 0;
    const std::string whole = "(u < " + std::to_string(NFULL) + " || col + EWF_VEC <= cols)";
    const std::string inside = ragged ? "if (u < " + std::to_string(NFULL) + " || col + e_ < cols) " : std::string("");
    auto emit_row_load = [&](int k, const std::string &ind, const std::string &dst) {
        const Operand &op = c.ops[k];
        std::string nm = opname(k);
        if (op.access == Access::Vector && loose) {
            if (ragged) {
                o << ind << "if " << whole << " " << dst << " = ewf_ld_u<" << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col);\n";
                o << ind << "else { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC - 1; ++e_) if (col + e_ < cols) " << dst << ".e[e_] = q_" << nm << "[col + e_]; }\n";
            }
            else o << ind << dst << " = ewf_ld_u<" << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col);\n";
        }
        else if (op.access == Access::Vector)
            o << ind << dst << " = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col);\n";
        else
            o << ind << "_Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) " << inside << dst << ".e[e_] = q_" << nm
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
        for (int k : row_ops) if (!late[k]) o << "        ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> x_" << opname(k) << "[" << U << "];\n";
        open_pass();
        for (int k : row_ops) if (!late[k]) emit_row_load(k, "            ", "x_" + opname(k) + "[u]");
        close_pass();
    }

    EmitCtx cx;
    cx.input = [&](int k) {
        if (c.ops[k].stride[in_d] == 0) return "ewf_in(g_" + opname(k) + ")";
        return resident && !late[k] ? "ewf_in(x_" + opname(k) + "[u].e[e_])" : "ewf_in(w_" + opname(k) + ".e[e_])";
    };
    cx.coord = [&](int d) {
        if (d == in_d) return std::string("col + e_");
        return "o" + std::to_string(d);
    };
    auto stream_loads = [&](const std::vector<char> &need) {
        for (int k : inputs_of(need)) {
            if (c.ops[k].stride[in_d] == 0 || (resident && !late[k])) continue;
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
        if (!fastn[l].empty()) {
            const std::string L = std::to_string(l), xr = "x_" + opname(fast_op[l]);
            const char *fold = nrows <= grid_cap ? "ewf_block_reduce_once" : "ewf_block_reduce";
            o << "        float rr_max" << L << "; int rr_arg" << L << ";\n        {\n";
            o << "        ewf_fmax fm_; fm_.m = ewf_bits_f32(0xff800000u); fm_.c = 0.0f;\n";
            open_pass();
            o << "            { float s_ = 0.0f;\n";
            o << "              _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
            if (ragged) o << "                if (u >= " << NFULL << " && col + e_ >= cols) continue;\n";
            o << "                const float t_ = ewf_in(" << xr << "[u].e[e_]);\n";
            o << "                fm_.m = __builtin_fmaxf(fm_.m, t_); s_ += t_;\n              }\n";
            o << "              fm_.c = __builtin_fmaf(s_, 0.0f, fm_.c); }\n";
            close_pass();
            o << "        const float tm_ = fm_.m;\n";
            o << "        fm_ = " << fold << "<EWF_NWAVES>(fm_, ewf_fmax_combine(), sm_fm" << L << ", tid);\n";
            o << "        if (fm_.c == fm_.c) {\n";
            // the same bits in every thread (each folds the same per-wavefront values in the same
            // order), so the branch is uniform across the workgroup
            o << "            int ix_ = 2147483647;\n";
            o << "            if (tm_ == fm_.m) {\n";
            o << "                #pragma unroll\n                for (int u = " << U - 1 << "; u >= 0; --u) {\n";
            o << "                    const idx_t col = (idx_t)(u * EWF_BLOCK + tid) * EWF_VEC;\n";
            o << "                    if (u >= " << NFULL << " && col >= cols) continue;\n";
            o << "                    _Pragma(\"unroll\") for (int e_ = EWF_VEC - 1; e_ >= 0; --e_) {\n";
            if (ragged) o << "                        if (u >= " << NFULL << " && col + e_ >= cols) continue;\n";
            o << "                        if (ewf_in(" << xr << "[u].e[e_]) == fm_.m) ix_ = (int)(col + e_);\n";
            o << "                    }\n                }\n            }\n";
            o << "            ix_ = " << fold << "<EWF_NWAVES>(ix_, ewf_imin(), sm_ix" << L << ", tid);\n";
            o << "            rr_max" << L << " = fm_.m; rr_arg" << L << " = ix_;\n";
            o << "        } else {\n";
            {
                // a NaN or an infinity somewhere in the row: the fold that ranks them
                std::string an = "AccS" + L, av = "accs" + L;
                std::vector<int> tg;
                for (int n : fastn[l]) tg.push_back(g.nodes[n].args[0]);
                std::vector<char> need = needed(tg);
                o << "        " << an << " " << av << " = " << an << "_identity();\n";
                open_pass();
                o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) {\n";
                if (ragged) o << "                if (u >= " << NFULL << " && col + e_ >= cols) continue;\n";
                emit_values(need, cx, "                ");
                emit_accumulate(av, fastn[l], [&](int node) { return argmax_index(node, cx.coord); }, "                ", true);
                o << "            }\n";
                close_pass();
                emit_first_index(av, fastn[l], "(idx_t)tid * EWF_VEC < cols", "tid * EWF_VEC", "        ");
                o << "        " << av << " = " << fold << "<EWF_NWAVES>(" << av << ", " << an << "_combine(), sm_accs" << L << ", tid);\n";
                o << "        {\n";
                emit_results(av, fastn[l], "        ");
                for (int n : fastn[l])
                    o << "        rr_" << (g.nodes[n].op == EWF_RARGMAX ? "arg" : "max") << L << " = r" << n << ";\n";
                // (an arg-max alone leaves the maximum unset, a maximum alone the index: neither is read)
                o << "        }\n";
            }
            o << "        }\n        }\n";
            for (int n : fastn[l])
                o << "        const " << (g.nodes[n].op == EWF_RARGMAX ? "int" : "float") << " r" << n << " = rr_"
                  << (g.nodes[n].op == EWF_RARGMAX ? "arg" : "max") << L << ";\n";
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
        if (ragged) o << "                if (u >= " << NFULL << " && col + e_ >= cols) continue;\n";
        emit_values(need, cx, "                ");
        emit_accumulate(av, lvl[l], [&](int node) { return argmax_index(node, cx.coord); }, "                ", true);
        o << "            }\n";
        close_pass();
        // every thread walks its columns in increasing order, starting at tid * EWF_VEC
        emit_first_index(av, lvl[l], "(idx_t)tid * EWF_VEC < cols", "tid * EWF_VEC", "        ");
        // (every level has a buffer of its own: without a loop over rows it is written once)
        o << "        " << av << " = " << (nrows <= grid_cap ? "ewf_block_reduce_once" : "ewf_block_reduce") << "<EWF_NWAVES>(" << av << ", "
          << an << "_combine(), sm_acc" << l << ", tid);\n";
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
        if (ragged) o << "                if (u >= " << NFULL << " && col + e_ >= cols) continue;\n";
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
            if (op.access == Access::Vector && loose) {
                if (ragged) {
                    o << "            if " << whole << " ewf_st_u<" << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col, y_" << nm << ");\n";
                    o << "            else { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC - 1; ++e_) if (col + e_ < cols) q_" << nm << "[col + e_] = y_" << nm << ".e[e_]; }\n";
                }
                else o << "            ewf_st_u<" << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col, y_" << nm << ");\n";
            }
            else if (op.access == Access::Vector)
                o << "            " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(q_" << nm << " + col, y_" << nm << ");\n";
            else
                o << "            _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) " << inside << "q_" << nm << "[(col + e_) * p.st_" << nm
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
            if (has_cross) emit_cross_partial("            ");
            o << "        }\n";
        }
    }
    o << "    }\n";

    o << "}\n";
    int cross_block = 256;
    if (has_cross) cross_block = emit_cross_finish(final_out_ops, nrows);

    // ---- launch geometry and argument block
    p.grid = std::max<int64_t>(1, std::min(nrows, grid_cap));
    p.lds_bytes = 0;
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
