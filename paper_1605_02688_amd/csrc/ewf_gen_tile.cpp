#include "ewf_gen.h"

namespace ewf {

// =========================================================================================
// Tile / TileReduce


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
    // (four where only narrow accesses are possible -- an odd row pitch, a misaligned view --
    // so that a thread still has 16 bytes in flight: sums over float32 rows of 50257, 52 -> 43 us;
    // softmax cross-entropy on them 92 -> 71 us; more than four is slower again)
    int narrowest = 4;
    for (const Operand &op : c.ops) if (op.stride[R - 1] != 0) narrowest = std::min(narrowest, isz(op.storage));
    // (element-wise kernels, which also store, gain only with 2-byte accesses: float16 with an
    // odd length 66 -> 53 us, float32 89 -> 92 us)
    const bool narrow = with_reduce ? VEC * narrowest < 16 : VEC * narrowest <= 2;
    const int U = e.opts.unroll > 0 ? e.opts.unroll : ((heavy >= 4 && !narrow) || small) ? 1 : narrow ? 4 : 2;
    // arithmetic-heavy expressions run best with larger workgroups (measured on the 21-op
    // float16 workload: 512 threads beat 256 by 4-8 %), streaming ones with 256
    int block = heavy >= 4 ? 512 : 256;
    if (small) { block = 64; while (block < 256 && items / block > 512) block *= 2; }
    if (e.opts.block_threads > 0) block = e.opts.block_threads;
    if (block % 64 || block > 1024) return fail("block_threads must be a multiple of 64, at most 1024");

    // ---- outputs by role
    std::vector<int> ew_out_ops, group_out_ops, final_out_ops;        // operand numbers
    const int nin = g.ninputs;
    // reductions over the kept axes of per-group values (the mean of per-row losses): folded by
    // the finish kernel, a single workgroup then
    const bool has_cross = with_reduce && !red.cross_nodes.empty();
    if (has_cross && red.max_depth > 1) return fail("chained reductions along the rows need the row-resident class");
    for (size_t k = nin; k < c.ops.size(); k++) {
        const Node &v = g.nodes[g.outputs[c.ops[k].index].value];
        const int vn = g.outputs[c.ops[k].index].value;
        if (has_cross && after_cross[vn]) { final_out_ops.push_back((int)k); continue; }
        bool group = with_reduce && ((v.bcast & red.axes) == red.axes);
        if (with_reduce && red.edepth[vn] >= 1 && !group) return fail("an output depends on a reduction and varies along the reduced axes; only the row-resident class covers that");
        (group ? group_out_ops : ew_out_ops).push_back((int)k);
    }

    // Vectors that assume element alignment only (see Plan::loose_vec): whole vectors of a row are
    // read and written wide wherever the row starts; a row that ends inside a vector has that
    // last vector handled element by element (`ragged`).
    const bool loose = p.loose_vec;
    const bool ragged = loose && c.extent[R - 1] % VEC != 0;
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
    // A kernel that both streams outputs and accumulates runs best with one trip per tile
    // (bias + ReLU + channel sums on float32 [128,64,112,112]: 7 tiles of 1792 per plane 133.2 us,
    // 2 tiles of 6272 135.6 us; its backward pass 197.7 against 202.6 us); pure reductions keep
    // four trips (fewer partial results and workgroups: 41 against 45 us on 268 MB).
    if (with_reduce && !ew_out_ops.empty() && c.total >= ((int64_t)1 << 22)) target = one_trip;
    // ... and from a quarter of a GB on, tiles of 128 KB (1 GB of float32 summed: 8192-element
    // tiles 6.4 TB/s, 32768-element tiles 6.85; 512 MB of float16: 6.25 against 6.5; no gain at
    // 128 MB and below, where there would be too few tiles)
    // (light accumulations only: with the rescaled exp-sum and an arg-max, 512 rows of 131072
    // float32 took 53.0 us with these tiles against 51.0 us with 8192-element ones)
    bool light = heavy == 0;
    for (int n : red.level_nodes) light = light && g.nodes[n].op != EWF_RARGMAX && g.nodes[n].op != kRSumExpShifted && g.nodes[n].op != kRSumSqCentred;
    if (with_reduce && ew_out_ops.empty() && light) {
        int in_sz = 4;
        for (int k = 0; k < nin; k++) in_sz = std::min(in_sz, isz(c.ops[k].storage));
        if (c.total * in_sz >= ((int64_t)1 << 28)) target = std::max<int64_t>(target, 131072 / in_sz);
    }
    // Reductions over the groups follow: with few partials per group (at most 32) a thread of the
    // finish kernel folds a whole group, and hundreds of groups are in flight at once -- as long
    // as that leaves enough tiles for the chip.
    if (has_cross) {
        int64_t per_group = 1, ngroups_ = 1;
        for (int d = 0; d < R; d++) (c.reduced[d] ? per_group : ngroups_) *= c.extent[d];
        // (softmax cross-entropy on float32 [512, 131072]: 16 tiles per row 52.2-53.0 us a step,
        // 8 tiles 48.6-50.1 us, 4 tiles 51.6-52.0 us, 2 tiles 56.8-57.4 us)
        const int64_t slots = 8;
        if (ngroups_ * slots >= (int64_t)4 * device_cu_count()) target = std::max(target, ceil_div(per_group, slots));
    }
    if (e.opts.tile_elems > 0) target = e.opts.tile_elems;
    {
        int64_t rem = target;
        for (int d = R - 1; d >= 0 && rem > 1; d--) {
            if (with_reduce && !c.reduced[d]) break;
            if (c.extent[d] <= rem) { T[d] = c.extent[d]; rem /= T[d]; continue; }
            int64_t n = ceil_div(c.extent[d], rem);
            int64_t t = ceil_div(c.extent[d], n);
            if (d == R - 1) {
                t = ceil_div(t, VEC) * VEC;
                // tiles that start on 128-byte lines: a line shared by two tiles is fetched (or
                // partially written) by two workgroups, usually on different dies (2092-element
                // float32 tiles ran 7 % slower than 1792-element ones)
                int min_sz = 4;
                for (const Operand &op : c.ops) min_sz = std::min(min_sz, isz(op.storage));
                const int64_t line = 128 / min_sz;
                if (t >= 4 * line && ceil_div(t, line) * line <= c.extent[d]) t = ceil_div(t, line) * line;
            }
            T[d] = t;
            break;
        }
    }
    if (loose) {
        // a tile holds whole vectors along the rows (its last one may reach past the row's end)
        if (T[R - 1] < VEC) return fail("rows too short for wide accesses");
        T[R - 1] = ceil_div(T[R - 1], VEC) * VEC;
    }
    // ---- permuted operands: stage through LDS
    // An operand whose own fastest dimension is not the output's would be read with one
    // narrow access per element.  Instead the workgroup reads the operand's part of the tile
    // along the operand's fastest dimension with wide accesses, scatters it into an LDS copy
    // of the tile laid out in the output's order, and the compute phase reads it back with
    // one wide LDS access per vector.  The tile is shaped so that both sides see long runs.
    int64_t stage_patch_a = 0;                         // pieces per index of the patch dimension (0: plain memory order)
    std::vector<int> stage_order;                      // digits of a staged piece's number, fastest first
    std::vector<int> staged;                           // operand numbers
    std::vector<int> sdims;                            // dims ordered by the staged operand's stride
    int VS = 1;
    if (!with_reduce && !e.opts.no_lds_staging && c.total >= 65536 && R >= 2 && !loose) {
        for (int k = 0; k < nin && staged.empty(); k++) {
            const Operand &op = c.ops[k];
            if (op.access != Access::Gather || !live[g.input_node[k]]) continue;      // (an input no output uses is never read)
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
        if (te * isz(c.ops[staged[0]].storage) > 40 * 1024) {
            block = 768;
            // ... unless that leaves a nearly empty last trip: eight wavefronts have the registers
            // to take such a trip's items along with the trip before (below), twelve have not
            // (reading "B" of the float16 stress workload, 49 wavefronts of items per tile: 768 threads
            // 91.7-93.0 us, 512 threads with the two last trips in one 89.7-90.0 us)
            auto last_fill = [&](int64_t b) { const int64_t s_ = b * VEC * U, n_ = ceil_div(te, s_); return (double)(te - (n_ - 1) * s_) / (double)s_; };
            if (e.opts.no_prefetch != 1 && last_fill(768) <= 0.25 && last_fill(512) <= 0.25) block = 512;
        }
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
        // Which 16-byte piece of the staged tile a lane loads.  Taken in the operand's memory
        // order, the 64 lanes of a wavefront may differ only along dimensions that are slow in the
        // LDS copy, and their scattered writes then fall into a few banks whatever the padding
        // (every lane writes the same position of the copy's fastest dimension: 82 % of the LDS's
        // active cycles were bank conflicts on reading "B" of the float16 stress workload).  So
        // a wavefront takes an 8 x 8 patch: eight neighbouring pieces in memory order (128
        // contiguous bytes where a run of the operand's fastest dimension holds eight) at each of
        // eight neighbouring indices of the copy's fastest dimension.  The pieces are numbered
        // with that dimension as the slowest digit to get there.
        {
            const int pd = R - 1;
            auto at = std::find(st.begin(), st.end(), pd);
            int64_t A = 1;
            for (int d : st) if (d != pd) A *= T[d];
            A /= VS;
            if (at != st.end() && pd != s0 && st.size() >= 2 && A % 8 == 0 && T[pd] % 8 == 0) {
                st.erase(at);
                st.push_back(pd);
                stage_patch_a = A;
            }
            stage_order = st;
        }
        auto piece_of = [&](int64_t q) {
            if (!stage_patch_a) return q;
            const int64_t b = q / 64, l = q % 64, na = stage_patch_a / 8;
            return (b % na) * 8 + (l & 7) + stage_patch_a * ((b / na) * 8 + (l >> 3));
        };
        auto conflicts = [&](int64_t pad) {
            // passes one scattered write of a wavefront needs: the LDS has 32 banks of 4 bytes
            // and takes the 64 lanes as two halves; a half needs as many passes as the largest
            // number of distinct words that fall into one bank
            int total = 0;
            for (int half = 0; half < 2; half++) {
                std::map<int64_t, std::vector<int64_t>> bank;
                for (int lane = half * 32; lane < half * 32 + 32; lane++) {
                    int64_t j = piece_of(lane) * VS, addr = 0;
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
        if (g.nodes[n].op == EWF_RARGMAX && ((!tiled.empty() && argmax_canon_dim(n) != tiled[0]) || argmax_rank(n) > 1)) ascending = false;
    std::vector<char> need = needed(targets);
    std::vector<int> used_inputs = inputs_of(need);

    emit_header(block);
    build_layout();
    if (with_reduce) emit_acc_struct("Acc", level);
    if (has_cross) emit_acc_struct("AccX", red.cross_nodes);
    std::vector<int> all_dims;
    for (int d = 0; d < R; d++) all_dims.push_back(d);
    std::vector<int> load_ops;                         // operand numbers read per element
    for (int k : used_inputs) load_ops.push_back(k);

    // what one trip of a thread holds in registers between its loads and its arithmetic
    // When the tile's last trip would be nearly empty (a few wavefronts with work, the others
    // waiting at the barrier for a whole round of memory latency), its items ride with the trip
    // before: those wavefronts issue both trips' loads together.
    const int64_t ntrips = ceil_div(TE, step);
    const bool prefetch = TE > step && !(e.opts.no_prefetch == 1 || (heavy >= 4 && e.opts.no_prefetch == 0));
    const bool fused_tail = !staged.empty() && !prefetch && e.opts.no_prefetch != 1 && U == 1 && block <= 512 && ntrips >= 2 && (TE - (ntrips - 1) * step) * 4 <= step;
    const int UI = fused_tail ? 2 : U;                 // items a thread may hold at once
    // (two items in flight take about a hundred registers: room for four wavefronts per SIMD, and
    // the register allocator is told so that it does not spill to keep more resident)
    if (fused_tail) auto_waves_per_simd = 4;
    o << "struct Item {\n    bool ok[" << UI << "];\n    int L[" << UI << "];\n";
    if (ragged) o << "    int nv[" << UI << "];\n";              // elements of the vector that lie inside the row
    for (int d : tiled) o << "    int c" << d << "[" << UI << "];\n";
    for (int k : load_ops) {
        const Operand &op = c.ops[k];
        if (op.access == Access::Splat && !is_staged(k)) o << "    " << ctype(op.storage) << " x_" << opname(k) << "[" << UI << "];\n";
        else o << "    ewf_vec<" << ctype(op.storage) << ", EWF_VEC> x_" << opname(k) << "[" << UI << "];\n";
    }
    o << "};\n";

    o << "extern \"C\" __global__ void __launch_bounds__(EWF_BLOCK) " << occupancy_attr() << "ewf_kernel(const Params p)\n{\n";
    o << "    const int tid = threadIdx.x;\n";
    std::string ind = "        ";
    // When every reduction group is a single tile the workgroup holds the whole group: it folds
    // its wavefronts through LDS and writes the results itself -- one launch, no workspace.
    bool one_tile = with_reduce;
    for (int d = 0; d < R; d++) if (c.reduced[d] && ntile[d] != 1) one_tile = false;
    if (has_cross) one_tile = false;
    // With reductions over the groups to follow and few tiles per group, a thread of the finish
    // kernel takes a whole group: the workgroup then leaves one partial per tile (its wavefronts
    // folded through LDS), stored with the group as the fastest index so that neighbouring threads
    // of the finish kernel read neighbouring partials.
    int64_t nslots_host = 1;
    for (int d = 0; d < R; d++) if (c.reduced[d]) nslots_host *= ntile[d];
    const bool cross_per_thread = has_cross && nslots_host <= 32;
    if (with_reduce && !one_tile) o << "    Acc *const partials = (Acc *)p.ws_partials;\n";
    // A kernel that also streams element-wise outputs takes one trip per tile and ends right after
    // it: folding its wavefronts through LDS first costs a wait for the slowest of them and leaves
    // the finish kernel a quarter of the partials (bias + ReLU + channel sums on float32
    // [128,64,112,112]: 133.3 -> 131.5 us a step, [128,256,56,56] 131.5 -> 130.4, [32,64,112,112]
    // 36.8 -> 36.0; its backward pass and pure reductions the same within 0.3 %).
    const bool wg_partials = with_reduce && !one_tile && !cross_per_thread && !ew_out_ops.empty() && TE <= step && block > 64;
    if (one_tile || cross_per_thread || wg_partials) o << "    __shared__ Acc sm_one[EWF_NWAVES];\n";
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
        // Two phases, so that the loads of up to eight trips are in flight together whatever the
        // compiler can prove about the bounds test: first every trip's load, unconditionally (a
        // piece outside the tile reads the tile's first piece instead), then the scattered LDS
        // writes of the pieces inside.  (With a branch around each load the trips ran one after
        // the other, a round trip to memory each: 5 % on the float16 stress workload.)
        const int64_t trips_ = ceil_div(TE, (int64_t)block * VS);
        const int64_t chunk_ = std::min<int64_t>(trips_, 8);
        o << ind << "for (int J00 = 0; J00 < " << TE << "; J00 += " << chunk_ * block * VS << ") {\n";
        o << ind << "    int slm_[" << chunk_ << "]; bool sk_[" << chunk_ << "];\n";
        for (int k : staged) o << ind << "    ewf_vec<" << ctype(c.ops[k].storage) << ", " << VS << "> sv_" << opname(k) << "[" << chunk_ << "];\n";
        o << ind << "    _Pragma(\"unroll\") for (int t_ = 0; t_ < " << chunk_ << "; ++t_) {\n";
        o << ind << "    const int J0 = J00 + t_ * " << (int64_t)block * VS << ";\n";
        if (stage_patch_a) {
            o << ind << "    int j_;\n";
            o << ind << "    { const int q_ = J0 / " << VS << " + tid, b_ = q_ >> 6, l_ = q_ & 63;    // an 8 x 8 patch of pieces per wavefront\n";
            const int64_t na_ = stage_patch_a / 8, nb_ = ceil_div(ceil_div(trips_, chunk_) * chunk_ * block, 64) + 1;
            o << ind << "      const int bq_ = " << div_small("b_", na_, nb_) << ", br_ = b_ - (int)ewf_mul24(bq_, " << na_ << ");\n";
            o << ind << "      j_ = (br_ * 8 + (l_ & 7) + " << stage_patch_a << " * (bq_ * 8 + (l_ >> 3))) * " << VS << "; }\n";
        } else {
            o << ind << "    int j_ = J0 + tid * " << VS << ";\n";
        }
        o << ind << "    bool k_ = J0 < " << TE << " && j_ < " << TE << ";\n";
        o << ind << "    int lm_ = 0; ioff_t g_ = 0;\n";
        const std::vector<int> &st = stage_order;      // the staged operand's dims with T > 1, fastest digit first
        int64_t jrange = TE;                           // what is left of j_ stays below this (for pieces inside the tile)
        for (size_t i = 0; i < st.size(); i++) {
            int d = st[i];
            if (i + 1 < st.size()) o << ind << "    { int c_; " << divmod_small("c_", "j_", T[d], jrange) << "\n";
            else o << ind << "    { const int c_ = j_;\n";
            jrange = ceil_div(jrange, T[d]);
            if (c.extent[d] % T[d]) o << ind << "      k_ = k_ && (o" << d << " + c_ < p.ext[" << d << "]);\n";
            o << ind << "      lm_ += c_ * " << LSP[d] << ";\n";
            if (d == s0) o << ind << "      g_ += (ioff_t)c_; }\n";
            else o << ind << "      g_ += " << product("c_", "p.st_" + opname(staged[0]) + "[" + std::to_string(d) + "]", c.ops[staged[0]].stride[d]) << "; }\n";
        }
        o << ind << "    sk_[t_] = k_; slm_[t_] = lm_;\n";
        o << ind << "    if (!k_) g_ = 0;\n";
        for (int k : staged) {
            const Operand &op = c.ops[k];
            // a staged operand is read exactly once through these wide loads: stream it past the
            // caches under the same rule as the unit-stride operands
            int64_t fp_ = isz(op.storage);
            for (int d = 0; d < R; d++) if (op.stride[d] != 0) fp_ *= c.extent[d];
            const bool nt_ = e.opts.streaming == 1 || (e.opts.streaming == 0 && fp_ >= ((int64_t)32 << 20));
            o << ind << "    sv_" << opname(k) << "[t_] = " << (nt_ ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", " << VS << ">(ewf_at(q_" << opname(k) << ", g_));\n";
        }
        o << ind << "    }\n";
        o << ind << "    _Pragma(\"unroll\") for (int t_ = 0; t_ < " << chunk_ << "; ++t_) {\n";
        o << ind << "        if (!sk_[t_]) continue;\n";
        for (int k : staged)
            o << ind << "        _Pragma(\"unroll\") for (int e_ = 0; e_ < " << VS << "; ++e_) lds_" << opname(k) << "[slm_[t_] + e_ * " << LSP[s0]
              << "] = sv_" << opname(k) << "[t_].e[e_];\n";
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
            int64_t lrange = TE;
            for (size_t i = 0; i < tiled.size(); i++) {
                int d = tiled[i];
                if (i + 1 < tiled.size()) { o << ind2 << "    " << divmod_small("it.c" + std::to_string(d) + "[u]", "l_", T[d], lrange) << "\n"; lrange = ceil_div(lrange, T[d]); }
                else o << ind2 << "    it.c" << d << "[u] = l_;\n";
                if (c.extent[d] % T[d]) o << ind2 << "    k_ = k_ && (o" << d << " + it.c" << d << "[u] < p.ext[" << d << "]);\n";
            }
        }
        if (ragged) {
            // (the distance to the row's end in the index type: it need not fit an int)
            o << ind2 << "    { const idx_t left_ = p.ext[" << in_d << "] - o" << in_d << " - (idx_t)it.c" << in_d << "[u];\n";
            o << ind2 << "      it.nv[u] = left_ < (idx_t)EWF_VEC ? (int)left_ : EWF_VEC; }\n";
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
                std::string pos = lds_pad ? "(L + " + div_small("L", LS[s0], TE) + " * " + std::to_string(lds_pad) + ")" : std::string("L");
                if (piece == VEC)
                    o << ind << "        it.x_" << nm << "[u] = ewf_ld<" << ctype(op.storage) << ", EWF_VEC>(&lds_" << nm << "[" << pos << "]);\n";
                else
                    o << ind << "        _Pragma(\"unroll\") for (int i_ = 0; i_ < " << VEC / piece << "; ++i_) ((ewf_vec<" << ctype(op.storage) << ", " << piece
                      << "> *)&it.x_" << nm << "[u])[i_] = ewf_ld<" << ctype(op.storage) << ", " << piece << ">(&lds_" << nm << "[" << pos << " + i_ * " << piece << "]);\n";
            }
            else if (op.access == Access::Vector && loose) {
                o << ind << "        { const " << ctype(op.storage) << " *const a_ = ewf_at(q_" << nm << ", " << offset_expr(k, false) << ");\n";
                if (ragged) {
                    o << ind << "          if (it.nv[u] == EWF_VEC) it.x_" << nm << "[u] = ewf_ld_u<" << ctype(op.storage) << ", EWF_VEC>(a_);\n";
                    o << ind << "          else { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC - 1; ++e_) if (e_ < it.nv[u]) it.x_" << nm << "[u].e[e_] = a_[e_]; } }\n";
                }
                else o << ind << "          it.x_" << nm << "[u] = ewf_ld_u<" << ctype(op.storage) << ", EWF_VEC>(a_); }\n";
            }
            else if (op.access == Access::Vector)
                o << ind << "        it.x_" << nm << "[u] = " << (op.stream ? "ewf_ld_nt<" : "ewf_ld<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << offset_expr(k, false) << "));\n";
            else if (op.access == Access::Splat)
                o << ind << "        it.x_" << nm << "[u] = *ewf_at(q_" << nm << ", " << offset_expr(k, true) << ");\n";
            else {
                o << ind << "        { const ioff_t b_ = " << offset_expr(k, false) << ";\n";
                o << ind << "          _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) " << (ragged ? "if (e_ < it.nv[u]) " : "") << "it.x_" << nm << "[u].e[e_] = *ewf_at(q_" << nm
                  << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm << "[" << in_d << "]); }\n";
            }
        }
    });
    const std::string text_c = capture([&]() {
        const std::string &ind = ind2;
        for (int k : ew_out_ops) o << ind << "    ewf_vec<" << ctype(c.ops[k].storage) << ", EWF_VEC> y_" << opname(k) << ";\n";
        // slots that take a vector of elements at once keep the element loop's values of their
        // argument and are folded after it
        std::vector<char> vslots(level.size(), 0), eslots(level.size(), 1);
        std::vector<int> vargs;
        if (with_reduce && VEC >= 2 && !e.opts.plain_extremes) {
            vslots = vector_slots(level, ascending);
            for (size_t i = 0; i < level.size(); i++) {
                if (!vslots[i]) continue;
                eslots[i] = 0;
                const int a = g.nodes[level[i]].args[0];
                if (std::find(vargs.begin(), vargs.end(), a) == vargs.end()) vargs.push_back(a);
            }
        }
        for (int a : vargs) o << ind << "    float xs" << a << "_[EWF_VEC]" << (ragged ? " = {}" : "") << ";\n";
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
        if (ragged) o << ind << "        if (e_ >= it.nv[u]) continue;\n";
        emit_values(need, cx, ind + "        ");
        if (with_reduce)
            emit_accumulate("acc", level, [&](int node) { return argmax_index(node, cx.coord); }, ind + "        ", ascending, &eslots);
        for (int a : vargs) o << ind << "        xs" << a << "_[e_] = v" << a << ";\n";
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            int v = g.outputs[op.index].value;
            const char *cv = op.storage == EWF_F16 ? "ewf_out_f16" : op.storage == EWF_I32 ? "ewf_out_i32" : "ewf_out_f32";
            o << ind << "        y_" << opname(k) << ".e[e_] = " << cv << "(v" << v << ");\n";
        }
        o << ind << "    }\n";
        for (int a : vargs)
            emit_vector_accumulate("acc", level, vslots, a, "xs" + std::to_string(a) + "_", ragged ? "it.nv[u] == EWF_VEC" : "",
                                   ragged ? "e_ >= it.nv[u]" : "", [&](int node) { return argmax_index(node, cx.coord); }, ind + "    ");
        for (int k : ew_out_ops) {
            const Operand &op = c.ops[k];
            std::string nm = opname(k);
            if (op.access == Access::Vector && loose) {
                o << ind << "    { " << ctype(op.storage) << " *const a_ = ewf_at(q_" << nm << ", " << offset_expr(k, false) << ");\n";
                if (ragged) {
                    o << ind << "      if (it.nv[u] == EWF_VEC) ewf_st_u<" << ctype(op.storage) << ", EWF_VEC>(a_, y_" << nm << ");\n";
                    o << ind << "      else { _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC - 1; ++e_) if (e_ < it.nv[u]) a_[e_] = y_" << nm << ".e[e_]; } }\n";
                }
                else o << ind << "      ewf_st_u<" << ctype(op.storage) << ", EWF_VEC>(a_, y_" << nm << "); }\n";
            }
            else if (op.access == Access::Vector)
                o << ind << "    " << (op.stream ? "ewf_st_nt<" : "ewf_st<") << ctype(op.storage) << ", EWF_VEC>(ewf_at(q_" << nm << ", " << offset_expr(k, false) << "), y_" << nm << ");\n";
            else {
                o << ind << "    { const ioff_t b_ = " << offset_expr(k, op.access == Access::Splat) << ";\n";
                o << ind << "      _Pragma(\"unroll\") for (int e_ = 0; e_ < EWF_VEC; ++e_) " << (ragged ? "if (e_ < it.nv[u]) " : "") << "*ewf_at(q_" << nm << ", b_ + (ioff_t)e_ * (ioff_t)p.st_" << nm
                  << "[" << in_d << "]) = y_" << nm << ".e[e_]; }\n";
            }
        }
    });

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
        if (fused_tail) {
            o << ind << "auto run_last_two = [&](const int L0) {\n";
            o << ind2 << "Item it;\n";
            o << ind2 << "#pragma unroll\n" << ind2 << "for (int u = 0; u < 2; ++u) {\n";
            o << text_a;
            o << ind2 << "    it.ok[u] = k_;\n";
            o << ind2 << "    if (k_) {\n" << text_b << ind2 << "    }\n" << ind2 << "}\n";
            o << ind2 << "#pragma unroll\n" << ind2 << "for (int u = 0; u < 2; ++u) {\n";
            o << ind2 << "    if (!it.ok[u]) continue;\n";
            o << text_c;
            o << ind2 << "}\n";
            o << ind << "};\n";
            if (ntrips > 2) o << ind << "for (int L0 = 0; L0 < " << (ntrips - 2) * step << "; L0 += " << step << ") run_item(L0);\n";
            o << ind << "run_last_two(" << (ntrips - 2) * step << ");\n";
        }
        else if (!looped) o << ind << "run_item(0);\n";
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
        } else if (cross_per_thread) {
            o << ind << "acc = ewf_block_reduce<EWF_NWAVES>(acc, Acc_combine(), sm_one, tid);\n";
            o << ind << "if (tid == 0) partials[(size_t)slot * (size_t)p.nrows + (size_t)group] = acc;\n";
        } else if (wg_partials) {
            o << ind << "acc = ewf_block_reduce<EWF_NWAVES>(acc, Acc_combine(), sm_one, tid);\n";
            o << ind << "if (tid == 0) partials[(size_t)group * (size_t)p.nslots + (size_t)slot] = acc;\n";
        } else {
            o << ind << "acc = ewf_wave_reduce(acc, Acc_combine());\n";
            o << ind << "if ((tid & 63) == 0) partials[((size_t)group * (size_t)p.nslots + (size_t)slot) * EWF_NWAVES + (tid >> 6)] = acc;\n";
        }
    }
    o << "    }\n}\n";

    if (with_reduce && !one_tile) {
        // one workgroup per group: a wavefront when a group has few partials, four otherwise
        int64_t nparts_host = wg_partials ? 1 : (int64_t)(block / 64);
        for (int d = 0; d < R; d++) if (c.reduced[d]) nparts_host *= ntile[d];
        // (1024 threads and eight partials in flight per thread when there are thousands: a total
        // over a large tensor is one group, and its finish is otherwise a chain of dependent loads)
        const int fin_block = nparts_host > 4096 ? 1024 : nparts_host > 256 ? 256 : 64;
        fin_block_out = fin_block;
        const int inflight = (int)std::min<int64_t>(8, std::max<int64_t>(1, ceil_div(nparts_host, fin_block)));
        if (has_cross) {
            int64_t ngroups_ = 1;
            for (int d = 0; d < R; d++) if (!c.reduced[d]) ngroups_ *= c.extent[d];
            if (ngroups_ > 8192) return fail("too many groups for the single-workgroup fold of a cross-group reduction");
            fin_block_out = emit_finish_all(level, group_out_ops, final_out_ops, cross_per_thread ? "p.nslots" : "p.nslots * EWF_NWAVES", ngroups_,
                                            gathers, cross_per_thread);
        }
        else emit_finish_lanes(level, group_out_ops, wg_partials ? "p.nslots" : "p.nslots * EWF_NWAVES", fin_block, inflight, gathers);
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
        p.workspace_bytes = (size_t)ngroups * (size_t)nslots * (size_t)(cross_per_thread || wg_partials ? 1 : block / 64) * acc_bytes(level);
        p.finish_grid = has_cross ? 1 : std::min<int64_t>(ngroups, (int64_t)1 << 20);
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


}  // namespace ewf
