// Internal data structures of the fused element-wise + reduce library (host side).
//
// Pipeline (paper section 2.2 reduced to one fused node): typed scalar graph -> frozen
// executable -> per-layout plan (canonical dimensions, kernel class, generated source,
// compiled code object) -> launch.
#pragma once

#include <cstdint>
#include <exception>
#include <map>
#include <memory>
#include <new>
#include <string>
#include <vector>

#include "ewf.h"

namespace ewf {

constexpr int kMaxDims = EWF_MAX_DIMS;

enum class NodeKind : int { Input, Scalar, Const, Iota, Apply, Cast, Reduce };

struct Node {
    NodeKind kind = NodeKind::Const;
    int op = 0;                 // Apply: ewf_op; Reduce: ewf_redop; Cast: target ewf_dtype
    int nargs = 0;
    int args[3] = {-1, -1, -1};
    int index = 0;              // Input / Scalar: ordinal; Iota: axis
    uint32_t axes = 0;          // Reduce: mask of reduced axes
    bool keep = false;          // Reduce: keep reduced axes in output shapes
    double cval = 0.0;          // Const
    // derived by the builder
    ewf_dtype vtype = EWF_F32;  // value type: EWF_F32 or EWF_I32
    ewf_dtype storage = EWF_F32;// Input: storage type
    uint32_t bcast = 0;         // bit d: value does not vary along d
    uint32_t dropped = 0;       // bit d: d is removed from the shape of an output of this value
    uint32_t in_dropped = 0;    // Input standing for a materialised reduction: the axes that reduction dropped
    int depth = 0;              // number of reduce nodes on the longest path from the inputs
};

struct OutputDecl {
    int value;
    ewf_dtype storage;
};

struct Graph {
    int ndim = 0;
    std::vector<Node> nodes;
    std::vector<OutputDecl> outputs;
    int ninputs = 0;
    int nscalars = 0;
    std::vector<int> input_node;   // node id of input k
    std::vector<int> scalar_node;  // node id of scalar k
};

// ---------------------------------------------------------------------------------------
// Canonical layout

enum class Access : int {
    Vector,   // unit stride along the innermost canonical dimension, aligned: one wide access
    Splat,    // stride 0 along the innermost dimension: one element repeated
    Gather,   // anything else: one access per element
    Staged    // gathered through an LDS tile filled along the operand's own fastest dimension
};

struct Operand {
    bool is_output = false;
    int index = 0;                    // input / output ordinal
    ewf_dtype storage = EWF_F32;
    uint32_t bcast = 0;               // original-rank mask (inputs: declared; outputs: value's)
    int64_t stride[kMaxDims] = {0};   // canonical, in elements
    uint64_t addr = 0;
    Access access = Access::Gather;
    bool stream = false;              // touched once and large: non-temporal accesses
    int alias_of = -1;                // outputs: operand number of the input it aliases exactly
};

// An operand as the caller passed it (original rank), for overlap checks.
struct RawView {
    uint64_t addr;
    int isz;
    int64_t ext[kMaxDims];
    int64_t str[kMaxDims];
    int rank;
};

struct Canon {
    int rank = 0;
    int64_t extent[kMaxDims] = {0};
    bool reduced[kMaxDims] = {false};     // member of the reduce axes of the fused reduction
    int orig_of_axis[kMaxDims];           // for iota: canonical dim that carries original axis d (-1: extent 1)
    int dim_of_axis[kMaxDims];            // canonical dim that original axis d went into (-1: extent 1)
    std::vector<Operand> ops;             // inputs then outputs
    int vec = 1;
    int vec_loose = 1;                    // the width that unit-stride operands would allow if neither the
                                          // alignment of their rows nor the row length had to fit it
    bool idx64 = false;
    bool byte32 = false;                  // every operand's byte span fits 32 bits
    int64_t total = 0;                    // product of extents
};

// ---------------------------------------------------------------------------------------
// Reduce structure of a graph (which kernel class can run it)

enum class KernelClass : int { None = 0, Tile = 1, TileReduce = 2, Row = 3, Col = 4, Multi = 5, Lane = 6 };

// A reduction the library introduces itself (never part of a caller's description):
// sum over the axes of exp(x - max over the same axes of x), accumulated in one pass as a
// (running maximum, sum relative to it) pair that is rescaled whenever the maximum grows.
// It turns the two chained reductions of a softmax or log-sum-exp into one level, so rows of
// any length can be split over workgroups.
constexpr int kRSumExpShifted = 64;
// Another one: sum over the axes of (x - mean of x over the same axes) squared, accumulated in
// one pass as a (count, running mean, sum of squared deviations) triple -- the published
// single-pass update for the variance, whose pairwise combine rule lets it fold across lanes,
// wavefronts and workgroups like any other accumulator.  It turns mean -> variance of the
// centred values (two chained reductions, two sweeps over memory) into one level.
constexpr int kRSumSqCentred = 65;

struct ReduceInfo {
    bool has_reduce = false;
    uint32_t axes = 0;                   // axes of the fused (first-level) reductions
    std::vector<int> level_nodes;        // reduce nodes over `axes` whose argument varies on them
    int max_depth = 0;                   // deepest chained level among level_nodes
    std::vector<int> cross_nodes;        // reductions of per-group values over the kept axes
    uint32_t cross_axes = 0;
    std::vector<int> edepth;             // per node: fused reductions on the longest path to it
    std::string unsupported;             // non-empty: why no single kernel covers the graph
};

struct KernelSource {
    std::string source;
    std::string entry;                   // kernel symbol
    std::string finish_entry;            // optional second kernel (empty if unused)
};

struct ParamField {
    enum Type { Ptr, I64, I32, F32 } type;
    std::string name;
    int count;
};

struct Plan;
struct Exec;
struct KernelTiming;                     // event pairs around the main kernels of timed runs (ewf_api.cpp)

// Packs kernel arguments with C layout rules for the struct the generator declares.
struct ParamLayout {
    std::vector<ParamField> fields;
    std::vector<size_t> offsets;
    size_t size = 0;
    void add(ParamField::Type t, const std::string &name, int count = 1);
    int find(const std::string &name) const;
    std::string declare(const std::string &struct_name, bool idx64) const;
};

// One kernel of a plan that needs several passes over memory: a sub-expression with its own
// executable, reading the caller's inputs and/or temporaries, writing temporaries and/or the
// caller's outputs.
struct Stage {
    std::unique_ptr<Exec> exec;
    std::vector<int> in_src;             // per stage input: >= 0 caller's input; < 0 temporary -(t+1)
    std::vector<int> out_dst;            // per stage output: >= 0 caller's output; < 0 temporary -(t+1)
    size_t ws_offset = 0, ws_bytes = 0;  // the stage's own workspace inside the caller's
};

struct Temp {
    ewf_dtype dtype = EWF_F32;
    int64_t shape[kMaxDims] = {0};
    int64_t strides[kMaxDims] = {0};
    size_t offset = 0, bytes = 0;        // place inside the caller's workspace
};

struct Plan {
    // Planning hints for the row class: refuse (EWF_EUNSUPPORTED, row_refused set) when a row
    // does not fit the registers of a workgroup or the rows are too few to occupy the chip, so
    // that the caller can try a plan in several passes first.
    bool avoid_poor_rows = false, row_refused = false;
    // Depth of the reduction chain once a max -> sum-of-exp pair has become one level: what a plan
    // in passes would have to sweep (one pass per level, and one for outputs that vary along the
    // rows).  A chain that stays two deep (mean, then variance of the centred values) costs such
    // a plan three sweeps, so rows that fit the registers at all stay with the row class.
    int fused_depth = 1;
    // Likewise for reductions over axes that are not neighbours in memory (a kept dimension lies
    // between them) with a short innermost run: the tile class would work on tiny tiles.  The
    // planner first tries two passes: one part of the axes (`split_first_axes`, original axis
    // mask: the outer ones in a column kernel, or the inner ones as short rows) and then the rest
    // on the much smaller result.
    bool avoid_short_runs = false, axes_refused = false;
    uint32_t split_first_axes = 0;
    KernelClass kclass = KernelClass::None;
    std::vector<Stage> stages;           // KernelClass::Multi only
    std::vector<Temp> temps;
    Canon canon;
    ReduceInfo red;
    ParamLayout layout;
    std::vector<uint8_t> args;           // packed argument block (pointers patched per run)
    std::vector<RawView> raw;            // the caller's views at planning time
    std::vector<char> may_be_null;       // operand may legally have a null pointer (empty)
    std::string source;
    std::vector<char> code;              // compiled code object
    void *function = nullptr;            // hipFunction_t, loaded on first launch
    int function_device = -1;
    int block = 256;
    int64_t grid = 0;
    void *finish_function = nullptr;     // second kernel folding partial results (0 grid: none)
    int64_t finish_grid = 0;
    int finish_block = 64;
    int lds_bytes = 0;
    int staged = 0;
    int64_t tile[kMaxDims] = {0};
    size_t workspace_bytes = 0;
    bool empty = false;                  // zero-size iteration space: nothing to traverse
    // The kernel was generated for canon.vec_loose: rows may start at any element and end inside
    // a vector.  Whole vectors are read and written with accesses that assume element alignment
    // only, the last vector of a row element by element.
    bool loose_vec = false;
    int strict_vec = 0;                  // canon.vec as the canonicaliser set it (0: not recorded yet)
    struct Fill { int output; int rank; int elem_bytes; uint32_t bits; };
    std::vector<Fill> fills;             // empty space: outputs that are reductions over an empty axis
    // empty space: values computed from such reductions.  The reductions are temporaries that a fill
    // kernel sets to the identity; one stage computes the outputs from them and the inputs.
    struct TempFill { int temp; uint32_t bits; };
    std::vector<TempFill> temp_fills;
    bool used_auto_occupancy = false;    // the generator asked for a register budget on its own
    bool no_auto_occupancy = false;      // ... and must not (it made the compiler spill)
};

struct Exec {
    bool is_stage = false;               // a stage of a multi-pass plan: must fit one kernel
    bool strict_rows = false;            // a stage that must not fall back on a poorly fitting row kernel
    // A stage may not read any input that fixes the extent of an axis it iterates over (it
    // reduces an index, say): the whole expression's extents, for the axes its own inputs leave open.
    bool has_forced_full = false;
    int64_t forced_full[kMaxDims] = {0};
    // Inputs (by index) that a later stage of the same plan reads again: such a tensor is loaded
    // with ordinary accesses so that the memory-side cache still holds it, or part of it.
    std::vector<char> read_again;
    Graph g;
    ewf_options opts{};
    int math_flavour = 1;                // 1 accurate, 2 native rate with fix-ups, 3 native rate
    bool auto_math = false;              // the flavour was chosen by the library (math_mode 0)
    std::map<std::string, std::unique_ptr<Plan>> plans;  // keyed by layout signature
    Plan *last = nullptr;
    int compile_count = 0;
    int nodes_before = 0, nodes_after = 0;   // size of the scalar graph before / after the rewrites
    KernelTiming *timing = nullptr;          // measurement aid; owned by the top-level executable, lent to stages
};

// ---- ewf_ir.cpp
// No C++ exception may cross the C ABI: every exported function runs its body through one of
// these.  Host memory running out is EWF_ENOMEM, anything else EWF_EINVAL with the exception's
// text as the error message (which is set without allocating where that is what failed).
void set_error_static(const char *text) noexcept;
void set_error_str(const std::string &s);
template <typename F>
ewf_status guarded(F &&body) noexcept
{
    try {
        return body();
    } catch (const std::bad_alloc &) {
        set_error_static("out of host memory");
        return EWF_ENOMEM;
    } catch (const std::exception &ex) {
        try { set_error_str(std::string("internal error: ") + ex.what()); } catch (...) { set_error_static("internal error"); }
        return EWF_EINVAL;
    } catch (...) {
        set_error_static("internal error");
        return EWF_EINVAL;
    }
}
// Test hook (ewf_debug_inject_fault): the points of the library where host memory is typically
// asked for call this; when armed on the calling thread it throws there.
void fault_point();
void arm_fault(int kind, int after);

void set_error(const char *fmt, ...);
const char *get_error();
ewf_status finalize_graph(Graph &g);     // recompute derived fields, validate outputs
// unit_mask: axes whose extent is 1 in this call (reducing over them is the identity)
ReduceInfo analyse_reductions(const Graph &g, uint32_t unit_mask);
void set_error_str(const std::string &s);
uint32_t all_mask(int ndim);

// ---- ewf_rewrite.cpp
// Merges duplicate nodes, folds constants, applies the stabilising rewrites; in place.
int rewrite_graph(Graph &g);
// Replaces every sum(exp(x - max(x))) over matching axes by one kRSumExpShifted node; in place.
// Returns the number of replacements.
// With `unless_argmax` a chain whose maximum is also the key of an arg-max stays as it is (the
// arg-max carries that maximum for free, so two sweeps over a row held in registers are cheaper).
int fuse_shifted_exp_sums(Graph &g, bool unless_argmax = false);
// Replaces every sum, product, max or min over exactly `axes` by the same reduction over `outer`
// (kept as broadcastable) followed by one over `axes` again, which then only folds the rest
// (reducing along an axis on which the argument is broadcastable is the identity).  In place;
// returns the number of reductions split, or -1 if the graph could not be rebuilt.
int split_reduction_axes(Graph &g, uint32_t axes, uint32_t outer);
// Replaces every sum over axes A of (x - m)^2 where m is the mean of x over A -- sum(x) over A times
// the literal 1/n or divided by the literal n, n the number of elements along A in this call
// (`full`: the extents) -- by one kRSumSqCentred node.  Returns the number of replacements.
int fuse_centred_squares(Graph &g, const int64_t *full);

// ---- ewf_canon.cpp
// Builds the canonical layout.  `in`/`out` give shapes and strides in the original rank
// (outputs: rank minus dropped axes).  Returns EWF_OK or an error (message set).
ewf_status canonicalize(const Exec &e, const ReduceInfo &red, const ewf_tensor *in, int nin,
                        const ewf_tensor *out, int nout, bool check_ptrs, Canon &c,
                        int64_t full_out[kMaxDims], std::vector<RawView> *raw_out = nullptr);
// Overlap rules between outputs and inputs / other outputs, on the caller's views.
ewf_status check_aliasing(const std::vector<RawView> &raw, int nin, int nout);
// `open_axes` (optional): extents for the axes that no input fixes (otherwise 1).
ewf_status infer_full_extents(const Graph &g, const ewf_tensor *in, int nin, int64_t full[kMaxDims],
                              const int64_t *open_axes = nullptr);

// ---- ewf_codegen.cpp
ewf_status generate(const Exec &e, Plan &p);

// ---- ewf_api.cpp
// With `lookup_only` a layout that has not been planned is an error (nothing is generated or compiled).
ewf_status make_plan(Exec &e, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout, Plan **result,
                     bool lookup_only = false);
// With `no_setup` the call only launches: a layout that has not been planned, or kernels that are
// not loaded on the current device yet, are errors instead of being compiled and loaded here.
ewf_status run_exec(Exec &x, const ewf_tensor *in, int32_t nin, const double *scalars, int32_t nscalars,
                    const ewf_tensor *out, int32_t nout, void *workspace, size_t workspace_bytes, void *hip_stream,
                    bool no_setup = false);
// Loads the kernels of a plan (of every stage of a plan in passes) on the current device.
ewf_status load_plan_functions(Plan &p);

// ---- ewf_multi.cpp
// Splits an expression that no single kernel class covers into stages: first-level reductions
// are materialised into temporaries, the rest of the graph reads them as broadcast operands.
// `g` is e.g or a rewritten copy of it with the same inputs, scalars and outputs.
// With `strict_rows` no stage may use the row class where it fits poorly (see Plan::avoid_poor_rows).
ewf_status plan_multi(Exec &e, const Graph &g, bool strict_rows, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout, Plan &plan);
// The iteration space is empty (some axis has extent 0) but the outputs `outs` are not: they are
// constant along every empty axis and computed from sums or products over one.  Plans one stage
// that reads those reductions as temporaries holding the identity.
ewf_status plan_empty_rest(Exec &e, const int64_t *full, const ewf_tensor *in, int nin, const ewf_tensor *out, int nout,
                           const std::vector<int> &outs, Plan &plan);
ewf_status run_multi(Exec &e, Plan &p, const ewf_tensor *in, int nin, const double *scalars, int nscalars,
                     const ewf_tensor *out, int nout, void *workspace, size_t workspace_bytes, void *hip_stream,
                     bool no_setup = false);

// ---- ewf_rtc.cpp
// Compiles HIP source for gfx950 (no device needed); identical sources share one code object.
ewf_status compile_source(const std::string &source, std::vector<char> &code, bool *was_cached);
// Loads `entry` from a code object on the current device (cached per device and code object).
ewf_status load_function(const std::vector<char> &code, const std::string &entry, void **function, int *device);
const char *prelude_source();
int device_cu_count();
void set_cache_dir(const char *path);
void cache_stats(int *mem_hits, int *disk_hits, int *compiles);
int64_t code_scratch_bytes(const std::vector<char> &code);
int peak_concurrent_compiles();

}  // namespace ewf

struct ewf_exec { ewf::Exec e; };
