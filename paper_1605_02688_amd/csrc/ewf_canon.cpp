// Broadcast / stride canonicaliser.
//
// The type of a variable fixes its rank and broadcastable pattern but neither its shape
// nor its strides (paper section 2.1.1), and transposes and basic slices are views
// (section 2.2.1, "Inplace").  This step turns what arrives at run time into the smallest
// equivalent description: broadcast dimensions become stride 0, extent-1 dimensions
// disappear, dimensions are ordered by memory stride, and neighbours that every operand
// walks contiguously are merged.  It then classifies each operand's access along the
// innermost dimension and picks the vector and index widths.
#include <algorithm>
#include <cstring>

#include "ewf_internal.h"

namespace ewf {

static int itemsize(ewf_dtype t) { return t == EWF_F16 ? 2 : 4; }

ewf_status infer_full_extents(const Graph &g, const ewf_tensor *in, int nin, int64_t full[kMaxDims], const int64_t *open_axes)
{
    if (nin != g.ninputs) { set_error("expected %d input tensor(s), got %d", g.ninputs, nin); return EWF_EINVAL; }
    if (nin > 0 && !in) { set_error("null input array"); return EWF_EINVAL; }
    for (int d = 0; d < kMaxDims; d++) full[d] = -1;
    for (int k = 0; k < nin; k++) {
        const Node &nd = g.nodes[g.input_node[k]];
        if (g.ndim > 0 && (!in[k].shape || !in[k].strides)) { set_error("input %d: null shape or strides", k); return EWF_EINVAL; }
        for (int d = 0; d < g.ndim; d++) {
            int64_t e = in[k].shape[d];
            if (e < 0) { set_error("input %d: negative extent", k); return EWF_EINVAL; }
            if (nd.bcast & (1u << d)) {
                if (e != 1) {
                    set_error("input %d: dimension %d is flagged broadcastable but has extent %lld", k, d, (long long)e);
                    return EWF_ESHAPE;
                }
            } else if (full[d] < 0) {
                full[d] = e;
            } else if (full[d] != e) {
                set_error("input %d: dimension %d has extent %lld, expected %lld (an unflagged dimension never broadcasts)",
                          k, d, (long long)e, (long long)full[d]);
                return EWF_ESHAPE;
            }
        }
    }
    for (int d = 0; d < g.ndim; d++) if (full[d] < 0) full[d] = open_axes ? open_axes[d] : 1;
    return EWF_OK;
}

static void byte_range(const RawView &v, uint64_t &lo, uint64_t &hi)
{
    int64_t span = 0;
    for (int d = 0; d < v.rank; d++) if (v.ext[d] > 1) span += (v.ext[d] - 1) * v.str[d];
    lo = v.addr;
    hi = v.addr + (uint64_t)(span + 1) * (uint64_t)v.isz;
}

// True if no two distinct coordinates of the view address the same element.
static bool self_disjoint(const RawView &v)
{
    std::vector<std::pair<int64_t, int64_t>> ds;   // (stride, extent)
    for (int d = 0; d < v.rank; d++) if (v.ext[d] > 1) ds.push_back({v.str[d], v.ext[d]});
    std::sort(ds.begin(), ds.end());
    int64_t reach = 0;                             // largest offset reachable with smaller strides
    for (auto &p : ds) {
        if (p.first <= reach) return false;
        reach += p.first * (p.second - 1);
    }
    return true;
}

// Lattice test for two views with identical strides: does a coordinate difference within
// the extents produce the element offset `delta`?
static bool lattice_hit(const std::vector<std::pair<int64_t, int64_t>> &ds, size_t i, int64_t delta)
{
    if (i == ds.size()) return delta == 0;
    int64_t s = ds[i].first, e = ds[i].second;
    int64_t q = delta / s;                          // try the two nearest multiples
    for (int64_t c = q - 1; c <= q + 1; c++) {
        if (c <= -e || c >= e) continue;
        if (lattice_hit(ds, i + 1, delta - c * s)) return true;
    }
    return false;
}

static bool views_overlap(const RawView &a, const RawView &b)
{
    // a view without elements overlaps nothing, whatever its pointer
    for (int d = 0; d < a.rank; d++) if (a.ext[d] == 0) return false;
    for (int d = 0; d < b.rank; d++) if (b.ext[d] == 0) return false;
    uint64_t alo, ahi, blo, bhi;
    byte_range(a, alo, ahi);
    byte_range(b, blo, bhi);
    if (ahi <= blo || bhi <= alo) return false;
    if (a.isz != b.isz || a.rank != b.rank) return true;
    std::vector<std::pair<int64_t, int64_t>> ds;
    for (int d = 0; d < a.rank; d++) {
        bool av = a.ext[d] > 1, bv = b.ext[d] > 1;
        if (!av && !bv) continue;
        if (av != bv || a.str[d] != b.str[d] || a.ext[d] != b.ext[d]) return true;   // conservative
        ds.push_back({a.str[d], a.ext[d]});
    }
    int64_t diff = (int64_t)(b.addr - a.addr);
    if (diff % a.isz) return true;
    std::sort(ds.begin(), ds.end(), [](auto &x, auto &y) { return x.first > y.first; });
    if (!self_disjoint(a)) return true;
    return lattice_hit(ds, 0, diff / a.isz);
}

static bool same_view(const RawView &a, const RawView &b)
{
    if (a.addr != b.addr || a.isz != b.isz) return false;
    for (int d = 0; d < a.rank; d++) {
        if (a.ext[d] != b.ext[d]) return false;
        if (a.ext[d] > 1 && a.str[d] != b.str[d]) return false;
    }
    return true;
}

ewf_status check_aliasing(const std::vector<RawView> &raw, int nin, int nout)
{
    for (int o = nin; o < nin + nout; o++) {
        for (int k = 0; k < o; k++) {
            if (!views_overlap(raw[k], raw[o])) continue;
            if (k < nin && same_view(raw[k], raw[o])) continue;
            set_error("%s %d overlaps output %d (only an exact alias of an input is allowed)",
                      k < nin ? "input" : "output", k < nin ? k : k - nin, o - nin);
            return EWF_EALIAS;
        }
    }
    return EWF_OK;
}

ewf_status canonicalize(const Exec &e, const ReduceInfo &red, const ewf_tensor *in, int nin,
                        const ewf_tensor *out, int nout, bool check_ptrs, Canon &c,
                        int64_t full[kMaxDims], std::vector<RawView> *raw_out)
{
    const Graph &g = e.g;
    const int nd = g.ndim;
    ewf_status st = infer_full_extents(g, in, nin, full, e.has_forced_full ? e.forced_full : nullptr);
    if (st != EWF_OK) return st;
    if (nout != (int)g.outputs.size()) { set_error("expected %d output tensor(s), got %d", (int)g.outputs.size(), nout); return EWF_EINVAL; }
    if (nout > 0 && !out) { set_error("null output array"); return EWF_EINVAL; }

    // ---- operands in the original rank
    std::vector<RawView> raw;
    c.ops.clear();
    for (int k = 0; k < nin; k++) {
        const Node &n = g.nodes[g.input_node[k]];
        Operand op;
        op.is_output = false; op.index = k; op.storage = n.storage; op.bcast = n.bcast;
        op.addr = (uint64_t)(uintptr_t)in[k].ptr;
        RawView rv{op.addr, itemsize(op.storage), {0}, {0}, nd};
        for (int d = 0; d < nd; d++) {
            int64_t s = (n.bcast & (1u << d)) ? 0 : in[k].strides[d];
            if (in[k].shape[d] <= 1) s = 0;
            if (s < 0) { set_error("input %d: negative strides are not supported", k); return EWF_EINVAL; }
            op.stride[d] = s;
            rv.ext[d] = in[k].shape[d]; rv.str[d] = s;
        }
        if (check_ptrs && !in[k].ptr) {
            bool empty = false;
            for (int d = 0; d < nd; d++) if (in[k].shape[d] == 0) empty = true;
            if (!empty) { set_error("input %d: null pointer", k); return EWF_EINVAL; }
        }
        c.ops.push_back(op);
        raw.push_back(rv);
    }
    bool out_nonempty = false;
    for (int k = 0; k < nout; k++) {
        const Node &v = g.nodes[g.outputs[k].value];
        Operand op;
        op.is_output = true; op.index = k; op.storage = g.outputs[k].storage; op.bcast = v.bcast;
        op.addr = (uint64_t)(uintptr_t)out[k].ptr;
        RawView rv{op.addr, itemsize(op.storage), {0}, {0}, nd};
        int od = 0;
        int orank = nd - __builtin_popcount(v.dropped);
        if (orank > 0 && (!out[k].shape || !out[k].strides)) { set_error("output %d: null shape or strides", k); return EWF_EINVAL; }
        bool nonempty = true;
        for (int d = 0; d < nd; d++) {
            rv.ext[d] = 1; rv.str[d] = 0; op.stride[d] = 0;
            if (v.dropped & (1u << d)) continue;
            int64_t want = (v.bcast & (1u << d)) ? 1 : full[d];
            int64_t have = out[k].shape[od], s = out[k].strides[od];
            od++;
            if (have != want) {
                set_error("output %d: dimension %d has extent %lld, expected %lld", k, d, (long long)have, (long long)want);
                return EWF_ESHAPE;
            }
            if (want == 0) nonempty = false;
            if (want <= 1) s = 0;
            if (s < 0) { set_error("output %d: negative strides are not supported", k); return EWF_EINVAL; }
            op.stride[d] = s; rv.ext[d] = want; rv.str[d] = s;
        }
        if (nonempty) out_nonempty = true;
        if (check_ptrs && nonempty && !out[k].ptr) { set_error("output %d: null pointer", k); return EWF_EINVAL; }
        if (nonempty && !self_disjoint(rv)) {
            set_error("output %d: distinct coordinates map to the same element", k);
            return EWF_EALIAS;
        }
        c.ops.push_back(op);
        raw.push_back(rv);
    }
    (void)out_nonempty;

    // ---- aliasing (section 2.2.1: an element-wise result may overwrite an input, exactly)
    if (check_ptrs) {
        st = check_aliasing(raw, nin, nout);
        if (st != EWF_OK) return st;
    }
    if (raw_out) *raw_out = raw;

    // ---- iteration space
    c.total = 1;
    for (int d = 0; d < nd; d++) c.total *= full[d];
    for (int d = 0; d < kMaxDims; d++) c.orig_of_axis[d] = c.dim_of_axis[d] = -1;
    if (c.total == 0) { c.rank = 0; return EWF_OK; }

    // which axes an iota node reads (they must keep their identity)
    uint32_t iota_axes = 0;
    for (const Node &n : g.nodes) {
        if (n.kind == NodeKind::Iota) iota_axes |= 1u << n.index;
        if (n.kind == NodeKind::Reduce && n.op == EWF_RARGMAX) iota_axes |= n.axes;   // the index it returns
    }

    // ---- drop extent-1 dimensions, order the rest by memory stride of a reference operand
    std::vector<int> dims;
    for (int d = 0; d < nd; d++) if (full[d] > 1) dims.push_back(d);
    auto varies_everywhere = [&](const Operand &op) {
        for (int d : dims) if (op.stride[d] == 0) return false;
        return true;
    };
    int ref = -1;
    for (int k = nin; k < nin + nout && ref < 0; k++) if (varies_everywhere(c.ops[k])) ref = k;
    if (ref < 0) {
        int best = -1;
        for (int k = 0; k < nin + nout; k++) {
            int cnt = 0;
            for (int d : dims) if (c.ops[k].stride[d] != 0) cnt++;
            if (cnt > best) { best = cnt; ref = k; }
        }
    }
    auto key = [&](int d) -> int64_t {
        if (ref >= 0 && c.ops[ref].stride[d] > 0) return c.ops[ref].stride[d];
        int64_t m = 0;
        for (const Operand &op : c.ops) m = std::max(m, op.stride[d]);
        return m;
    };
    std::stable_sort(dims.begin(), dims.end(), [&](int a, int b) { return key(a) > key(b); });

    // ---- merge neighbours that every operand walks contiguously
    struct CD { int64_t ext; bool red; bool iota; int orig; std::vector<int64_t> st; std::vector<int> origs; };
    std::vector<CD> cd;
    for (int d : dims) {
        CD x; x.ext = full[d]; x.red = (red.axes >> d) & 1u; x.iota = (iota_axes >> d) & 1u; x.orig = d;
        x.origs.push_back(d);
        for (const Operand &op : c.ops) x.st.push_back(op.stride[d]);
        cd.push_back(x);
    }
    for (int i = (int)cd.size() - 2; i >= 0; i--) {
        CD &a = cd[i], &b = cd[i + 1];
        bool ok = (a.red == b.red) && !a.iota && !b.iota;
        for (size_t k = 0; ok && k < a.st.size(); k++) ok = (a.st[k] == b.st[k] * b.ext);
        if (!ok) continue;
        b.ext *= a.ext;
        b.origs.insert(b.origs.end(), a.origs.begin(), a.origs.end());
        cd.erase(cd.begin() + i);
    }
    if (cd.empty()) {                       // a single element
        CD x; x.ext = 1; x.red = false; x.iota = false; x.orig = -1;
        x.st.assign(c.ops.size(), 0);
        cd.push_back(x);
    }
    if ((int)cd.size() > kMaxDims) { set_error("rank too large"); return EWF_EINVAL; }
    c.rank = (int)cd.size();
    for (int i = 0; i < c.rank; i++) {
        c.extent[i] = cd[i].ext;
        c.reduced[i] = cd[i].red;
        if (cd[i].orig >= 0 && cd[i].iota) c.orig_of_axis[cd[i].orig] = i;
        for (int o : cd[i].origs) c.dim_of_axis[o] = i;
        for (size_t k = 0; k < c.ops.size(); k++) c.ops[k].stride[i] = cd[i].st[k];
    }
    for (size_t k = 0; k < c.ops.size(); k++)
        for (int i = c.rank; i < kMaxDims; i++) c.ops[k].stride[i] = 0;

    // ---- index width (section 3.1.5: 64-bit indexing exists but 32-bit is faster)
    int64_t max_off = c.total;
    for (const Operand &op : c.ops) {
        int64_t off = 0;
        for (int i = 0; i < c.rank; i++) off += (c.extent[i] - 1) * op.stride[i];
        max_off = std::max(max_off, off);
    }
    c.idx64 = e.opts.force_index64 || max_off >= ((int64_t)1 << 31) - 65536;
    c.byte32 = !c.idx64 && max_off < ((int64_t)1 << 30) - 65536;

    // ---- vector width and access class along the innermost dimension
    const int in_d = c.rank - 1;
    int min_isz = 4;
    bool any_unit = false;
    for (const Operand &op : c.ops) if (op.stride[in_d] == 1) { any_unit = true; min_isz = std::min(min_isz, itemsize(op.storage)); }
    int vec = any_unit ? 16 / min_isz : 1;
    if (e.opts.force_scalar) vec = 1;
    auto vec_ok = [&](int v) {
        if (c.extent[in_d] % v) return false;
        for (const Operand &op : c.ops) {
            if (op.stride[in_d] != 1) continue;
            int bytes = std::min(16, v * itemsize(op.storage));
            if (op.addr % bytes) return false;
            for (int i = 0; i < in_d; i++) if (op.stride[i] % v) return false;
        }
        return true;
    };
    c.vec_loose = vec;
    while (vec > 1 && !vec_ok(vec)) vec /= 2;
    c.vec = vec;
    // what the launch moves through operands that are touched once: from 64 MiB on (twice the
    // level-two caches of all dies together) nothing of it is still cached when its turn comes again
    int64_t moved_once = 0;
    for (const Operand &op : c.ops) {
        int64_t footprint = itemsize(op.storage);
        bool once = true;
        for (int i = 0; i < c.rank; i++) { if (op.stride[i] != 0) footprint *= c.extent[i]; else if (!(op.is_output && c.reduced[i])) once = false; }
        if (once || op.is_output) moved_once += footprint;
    }
    for (Operand &op : c.ops) {
        if (op.stride[in_d] == 1 || c.extent[in_d] == 1) op.access = Access::Vector;
        else if (op.stride[in_d] == 0) op.access = Access::Splat;
        else op.access = Access::Gather;
        if (c.extent[in_d] == 1 && op.stride[in_d] == 0) op.access = Access::Splat;
        // streaming hint: every element is touched once and the operand is far larger than
        // what the caches could keep for a later consumer
        int64_t footprint = itemsize(op.storage);
        bool once = true;
        for (int i = 0; i < c.rank; i++) { if (op.stride[i] != 0) footprint *= c.extent[i]; else if (!(op.is_output && c.reduced[i])) once = false; }
        if (op.is_output) once = true;
        op.stream = op.access == Access::Vector && once &&
                    (e.opts.streaming == 1 ||
                     (e.opts.streaming == 0 && (footprint >= ((int64_t)32 << 20) || (moved_once >= ((int64_t)64 << 20) && footprint >= ((int64_t)4 << 20)))));
        // ... unless a later stage of the plan reads the tensor again: a non-temporal load would not
        // leave it in the 256 MB memory-side cache.  Ordinary loads are slower in a kernel that only
        // reads (a sum over 268 MB: 47.6 against 44.9 us), but what the later stage then finds
        // cached outweighs that, also for tensors larger than the cache, of which a part survives
        // (batch normalisation over axis 0, statistics then the normalised tensor, rotating
        // buffers: float16 [65536, 1024] 87.3 -> 83.6 us, float32 [32768, 1024] 77.9 -> 72.1 us,
        // [65536, 1024] (268 MB) 138.4 -> 132.3 us, [131072, 1024] 269.0 -> 255.8 us, [262144, 1024]
        // (1.07 GB) 534.1 -> 526.9 us; not tried beyond)
        const size_t k_ = (size_t)(&op - c.ops.data());
        if (e.opts.streaming == 0 && !op.is_output && k_ < e.read_again.size() && e.read_again[k_] && footprint <= ((int64_t)1 << 30))
            op.stream = false;
    }
    return EWF_OK;
}

}  // namespace ewf
