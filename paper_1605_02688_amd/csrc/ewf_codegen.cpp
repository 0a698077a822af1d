// HIP source generator.
//
// One kernel per (expression, storage types, canonical layout class, vector width, index
// width); extents, strides and run-time scalars are kernel arguments so that a new shape of
// the same class reuses the compiled code (paper section 5.3 argues for passing such
// information at run time instead of baking it into generated modules; section 2.2.3
// describes per-node code generation, which here becomes per-fused-expression).
//
// Kernel skeletons, all written for 64-lane wavefronts (ewf_gen.h holds what they share, one
// source file each: ewf_gen_tile.cpp, ewf_gen_row.cpp, ewf_gen_col.cpp):
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
//   Col         reduced axes that are not the fastest-varying ones: lanes along the innermost
//               kept dimension, rows spread over wavefronts and workgroups.
//   Lane        short rows: several rows per wavefront, a power-of-two group of lanes each
//               (ewf_gen_lane.cpp).
#include "ewf_gen.h"

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

void finish_layout(ParamLayout &L)
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


// =========================================================================================

ewf_status generate(const Exec &e, Plan &p)
{
    // The tile and row classes can use wide accesses on rows that start at any element and end inside a
    // vector (an odd row pitch -- a vocabulary of 50257 --, a view that begins at an odd
    // element): softmax cross-entropy statistics on [1280, 50257] 73 us element by element.
    // Element-wise kernels gain only where the strict width leaves 2-byte accesses (float16 of odd
    // length 53 -> 48 us, a float16 view from an odd element 66 -> 49 us; float32 streams as well
    // element by element: 89 us against 101 us with the checks that rows ending inside a vector need).
    // (a plan can come here more than once -- another class after a refusal, the same class again
    // without a register hint that made the compiler spill -- so every call starts from the
    // canonicaliser's width)
    if (p.strict_vec == 0) p.strict_vec = p.canon.vec;
    p.canon.vec = p.strict_vec;
    p.loose_vec = false;
    const Canon &c = p.canon;
    int narrowest = 4;
    for (const Operand &op : c.ops) if (op.stride[c.rank - 1] != 0) narrowest = std::min(narrowest, op.storage == EWF_F16 ? 2 : 4);
    const bool worth = p.kclass == KernelClass::TileReduce || p.kclass == KernelClass::Row ||
                       (p.kclass == KernelClass::Tile && c.vec * narrowest <= 2);
    if (worth && c.vec_loose > c.vec && !e.opts.force_scalar && c.extent[c.rank - 1] >= 4 * c.vec_loose) {
        const int strict = c.vec;
        p.canon.vec = c.vec_loose;
        p.loose_vec = true;
        Gen wide(e, p);
        ewf_status st = p.kclass == KernelClass::Row ? wide.gen_row() : wide.gen_tile(p.kclass == KernelClass::TileReduce);
        if (st == EWF_OK) return st;
        p.canon.vec = strict;
        p.loose_vec = false;
    }
    Gen gen(e, p);
    switch (p.kclass) {
    case KernelClass::Tile: return gen.gen_tile(false);
    case KernelClass::TileReduce: return gen.gen_tile(true);
    case KernelClass::Row: return gen.gen_row();
    case KernelClass::Col: return gen.gen_col();
    case KernelClass::Lane: return gen.gen_lane();
    default: set_error("no kernel class"); return EWF_EUNSUPPORTED;
    }
}

}  // namespace ewf
