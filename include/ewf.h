/*
 * ewf.h -- C ABI of the fused element-wise + reduce library for MI355X (gfx950).
 *
 * The library evaluates, in ONE pass over n-d tensors, a directed acyclic graph of scalar
 * operations (the result of the paper's "Specialize" stage, section 2.2.1: successive
 * element-wise operations fused so the tensor is traversed once), with the typing rules of
 * section 2.1.1 (data type, rank and broadcastable pattern belong to a variable's type;
 * shape and strides do not) and the strided views of section 2.2.1 "Inplace" (transposes
 * and basic slices are views).  Reductions over chosen axes (sum, max, min, prod, arg-max)
 * are fused into the same pass.
 *
 * Life cycle, following section 2.2 (describe symbolically, compile once, call many times):
 *   ewf_graph_create -> ewf_input / ewf_scalar / ewf_const / ewf_iota / ewf_apply / ewf_cast /
 *   ewf_reduce / ewf_output      describe the typed scalar graph            (host only)
 *   ewf_compile                   type-check, freeze into an executable      (host only)
 *   ewf_plan                      canonicalise shapes/strides, generate and compile the
 *                                 gfx950 kernel for this layout class, cache it (no launch)
 *   ewf_run                       launch on the caller's stream              (asynchronous)
 *   ewf_run_static                the same without a caller's workspace      (asynchronous)
 *
 * Conventions
 *   - Every function returns 0 (EWF_OK) or a negative ewf_status.  No C++ exception crosses
 *     this boundary.  ewf_last_error() gives a thread-local message for the last failure on
 *     the calling thread (including the run-time compiler's log), valid until the next call.
 *   - Value ids are >= 0; a negative return from a graph-building call is an ewf_status.
 *   - All tensors of one graph have the same rank `ndim` (<= EWF_MAX_DIMS).  A dimension
 *     flagged broadcastable must have extent 1; an unflagged one must have the full extent
 *     of the iteration space, otherwise EWF_ESHAPE (the pattern is a guarantee, section 2.1.1).
 *   - Strides are in ELEMENTS, must be >= 0.  Shapes/strides arrays are host memory, read
 *     during the call only.
 *   - `ptr` members are DEVICE pointers owned by the caller: inputs, outputs and workspace.
 *     ewf_run neither allocates, frees nor synchronises (section 3.1.3: freeing device memory
 *     synchronises, so the hot path must not).
 *   - An output may alias an input only exactly (same pointer, shape and strides; section
 *     2.2.1: element-wise operations may overwrite an input); any other overlap between an
 *     output and an input or another output is EWF_EALIAS.
 *   - A tensor with a zero extent is legal: success, nothing traversed.  A sum or a product
 *     over an empty axis is 0 or 1, also inside an expression; a maximum, minimum or arg-max over
 *     an empty axis (or anything computed from one) is EWF_ESHAPE.
 *   - Thread safety: different ewf_exec handles may be used concurrently; one handle must be
 *     externally synchronised.
 */
#ifndef EWF_H
#define EWF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define EWF_MAX_DIMS 8

typedef int32_t ewf_status;
enum {
    EWF_OK = 0,
    EWF_EINVAL = -1,        /* malformed argument or graph                                  */
    EWF_ETYPE = -2,         /* value/storage type rule violated                             */
    EWF_ESHAPE = -3,        /* shape does not match the broadcastable pattern               */
    EWF_EALIAS = -4,        /* output overlaps an input or another output                   */
    EWF_ECOMPILE = -5,      /* run-time compilation failed (log in ewf_last_error)          */
    EWF_EHIP = -6,          /* a HIP runtime call failed                                    */
    EWF_ENOMEM = -7,        /* host allocation failed or workspace too small                */
    EWF_EUNSUPPORTED = -8   /* graph/layout combination no kernel class covers              */
};

/* Storage types of tensors; value types of scalar nodes are EWF_F32 or EWF_I32 only
 * (float16 is a storage format: it is widened to float32 on load, rounded to nearest even
 * on store; section 3.1.5 of the paper: half-precision storage in the new back-end). */
typedef enum { EWF_F32 = 0, EWF_F16 = 1, EWF_I32 = 2 } ewf_dtype;

/* Scalar operations.  Arithmetic needs operands of equal value type; there is no implicit
 * promotion (use ewf_cast).  Comparisons return int32 0/1.  EWF_WHERE(c,a,b) = a if c != 0
 * (a NaN condition counts as true) else b.  EWF_MAX / EWF_MIN propagate NaN. */
typedef enum {
    EWF_ADD = 0, EWF_SUB, EWF_MUL, EWF_DIV, EWF_NEG, EWF_ABS, EWF_EXP, EWF_LOG, EWF_LOG1P,
    EWF_SQRT, EWF_TANH, EWF_SIGMOID, EWF_MAX, EWF_MIN, EWF_POW, EWF_WHERE, EWF_GT, EWF_GE,
    EWF_LT, EWF_LE, EWF_EQ, EWF_NE, EWF_EXPM1, EWF_SQR, EWF_RECIP, EWF_OP_COUNT
} ewf_op;

/* Reductions.  EWF_RARGMAX returns the int32 index of the first occurrence of the maximum (a NaN
 * ranks above every number): along one axis the coordinate, over several axes the position in
 * their row-major order, taken in axis order (fewer than 2^31 positions). */
typedef enum { EWF_RSUM = 0, EWF_RMAX, EWF_RMIN, EWF_RPROD, EWF_RARGMAX } ewf_redop;

typedef int32_t ewf_value;
typedef struct ewf_graph ewf_graph;
typedef struct ewf_exec ewf_exec;

/* Compile options; zero-initialise for defaults. */
typedef struct {
    int32_t math_mode;      /* 1 accurate float32 routines (about one unit in the last place);
                               2 native-rate exp2/log2/rcp with fix-ups that keep log1p, expm1
                               and tanh relatively accurate near zero; 3 native-rate without
                               them (absolute error near zero about 6e-8); 0 auto: 3 iff every
                               output is stored as float16, else 1 -- except for values that
                               reach the outputs only as terms of a float32 sum, which use 2
                               (worst-case relative error of a term under 6e-6, inside the 1e-5
                               bar of reduction outputs), and for sigmoid and tanh, which use 2
                               wherever they do not feed a product, an extreme value, an
                               arg-max, a comparison or a conversion to an integer (bounded
                               results: relative error under 1.5e-6, absolute under 1.2e-7,
                               inside the 2e-6 / 1e-6 bar of element-wise outputs)             */
    int32_t force_scalar;   /* 1: never use vector (multi-element) memory accesses           */
    int32_t force_index64;  /* 1: 64-bit offset arithmetic even when 32 bits suffice         */
    int32_t block_threads;  /* 0 = library default                                           */
    int32_t unroll;         /* vectors per thread per tile; 0 = library default              */
    int32_t max_blocks;     /* cap on the grid; 0 = library default                          */
    int32_t no_lds_staging; /* 1: never stage permuted operands through LDS                  */
    int32_t streaming;      /* non-temporal accesses for operands touched once: 0 auto (operands
                               of 32 MiB or more), 1 always, 2 never                          */
    int32_t tile_elems;     /* elements per tile (per workgroup and loop trip); 0 = default  */
    int32_t waves_per_simd; /* register budget hint: resident wavefronts per SIMD to aim for
                               (1..8); 0 = compiler default                                   */
    int32_t no_prefetch;    /* the next trip's loads ahead of the current trip's arithmetic:
                               0 automatic, 1 never (nor a nearly empty last trip taken along
                               with the trip before it), 2 always                              */
    int32_t xcd_remap;      /* 1: neighbouring tiles go to the same accelerator die, whose L2
                               they then share (default 0: workgroup w takes tile w, which
                               measured faster on streaming workloads)                       */
    int32_t no_rewrite;     /* 1: compile the scalar graph as described (default: duplicates
                               merged, constants folded, log(1+x) -> log1p(x), exp(x)-1 ->
                               expm1(x), x*x and pow(x,2) -> a square, identities removed)   */
    int32_t split_rows;     /* chained reductions along rows (softmax, log-sum-exp): one workgroup
                               per row holding the row in registers, or several passes with the
                               rows split over workgroups (max -> sum of exp fused into one
                               level that is rescaled as the maximum grows).  0 automatic: split
                               when a row does not fit the registers or the rows are too few to
                               occupy the chip; 1 always split; 2 never                       */
    int32_t plain_extremes; /* 1: maxima, arg-maxima and sums of shifted exponentials are always
                               folded element by element with the rules that rank NaN (default
                               0: rows held in registers take the hardware maximum first and find
                               the index afterwards, streaming kernels fold a vector of finite
                               values at once; both fall back on those rules only for rows or
                               vectors that hold a NaN or an infinity)                         */
    int32_t reserved[1];
} ewf_options;

/* A strided n-d view of caller-owned device memory.  rank is implied by the graph (inputs:
 * ndim; outputs: ndim minus the axes dropped by reductions, see ewf_reduce). */
typedef struct {
    void *ptr;                /* device pointer                                             */
    const int64_t *shape;     /* host array, extents                                        */
    const int64_t *strides;   /* host array, element strides                                */
} ewf_tensor;

/* ---- graph description (host only; section 2.1.1: typed variables, apply nodes, SSA) ---- */

/* Creates an empty graph whose tensors all have rank ndim (0..EWF_MAX_DIMS). */
ewf_status ewf_graph_create(int32_t ndim, ewf_graph **g);
void ewf_graph_destroy(ewf_graph *g);

/* Tensor input number k (k counts ewf_input calls).  bcast_flags: ndim bytes, non-zero =
 * the dimension is broadcastable (extent 1, value repeated along it). */
ewf_value ewf_input(ewf_graph *g, ewf_dtype storage, const uint8_t *bcast_flags);
/* Run-time scalar number k (k counts ewf_scalar calls), passed by value to ewf_run so that
 * changing it needs no recompilation (section 5.3: pass information at run time instead of
 * hard-coding it in generated code).  dtype: EWF_F32 or EWF_I32. */
ewf_value ewf_scalar(ewf_graph *g, ewf_dtype dtype);
/* Literal baked into the kernel; rounded to dtype (EWF_F32 or EWF_I32). */
ewf_value ewf_const(ewf_graph *g, ewf_dtype dtype, double value);
/* int32 coordinate along `axis` of the iteration space. */
ewf_value ewf_iota(ewf_graph *g, int32_t axis);
/* Applies a scalar operation point-wise. */
ewf_value ewf_apply(ewf_graph *g, ewf_op op, const ewf_value *args, int32_t nargs);
/* Explicit conversion: to EWF_F32 (int32 -> float32, nearest even; float32 -> itself),
 * to EWF_F16 (rounds the value to the nearest float16, result stays a float32 value),
 * to EWF_I32 (truncation toward zero, saturating, NaN -> 0). */
ewf_value ewf_cast(ewf_graph *g, ewf_value v, ewf_dtype to);
/* Folds v over `axes` (numbered in the rank-ndim space).  The result is broadcastable along
 * the reduced axes and can be combined with full-rank values.  With keep_as_bcast == 0 the
 * reduced axes are removed from the shape of any output computed from the result alone. */
ewf_value ewf_reduce(ewf_graph *g, ewf_redop op, ewf_value v, const int32_t *axes, int32_t naxes,
                     int32_t keep_as_bcast);
/* Reverse-mode differentiation (section 2.1.3 of the paper: gradients are built symbolically
 * by traversing the graph from the outputs back to the inputs).  y[k] are float32 values of
 * the graph and ybar[k] their cotangents (float32 values of the same graph, usually further
 * inputs; a cotangent may be broadcastable where its value is not).  For every wrt[j] (a
 * float32 value, usually an input) the call appends the nodes of
 *     grads[j] = sum_k sum_elements ybar[k] * d y[k] / d wrt[j]
 * to the graph and returns their ids; declare them as outputs like any other value.  Where
 * wrt[j] is broadcastable and the cotangent is not, the result is summed over those axes (kept
 * as broadcastable, so it has the shape of wrt[j]).  Conventions: max/min give the cotangent to
 * the first operand on ties, reduce-max/min to every element equal to the result, abs has
 * derivative 0 at 0, comparisons and int32 values stop the cotangent, float16 rounding passes
 * it through; the derivative of a product reduction is the product of the other elements
 * (exact also where elements are zero). */
ewf_status ewf_grad(ewf_graph *g, const ewf_value *y, const ewf_value *ybar, int32_t ny,
                    const ewf_value *wrt, int32_t nwrt, ewf_value *grads);
/* Declares output number k (k counts ewf_output calls) stored as `storage`. */
ewf_status ewf_output(ewf_graph *g, ewf_value v, ewf_dtype storage);

/* ---- compile / plan / run (section 2.2: compile once into a callable) ---- */

/* Directory for compiled kernels kept across processes (section 2.2.3 of the paper: generated
 * code is cached on disk so that it is compiled once).  One file per kernel source, named by a
 * hash of the device helpers, the generated text, the compiler options and the run-time
 * compiler's version; written through a temporary file and a rename, so concurrent processes may
 * share a directory.  NULL or "" turns the disk cache off (the default; the in-process cache is
 * always on).  Also read from the environment variable EWF_CACHE_DIR when the library loads.
 * A directory that cannot be written is not an error: kernels are then compiled every time. */
ewf_status ewf_set_cache_dir(const char *path);

/* Type-level compilation.  opts may be NULL.  The graph may be destroyed afterwards. */
ewf_status ewf_compile(const ewf_graph *g, const ewf_options *opts, ewf_exec **out);
void ewf_exec_destroy(ewf_exec *e);

/* Shape inference for caller-side allocation: given the input tensors (ptr ignored), writes
 * rank and extents of output k.  shape_out must hold EWF_MAX_DIMS entries. */
ewf_status ewf_output_shape(ewf_exec *e, const ewf_tensor *in, int32_t nin, int32_t k,
                            int32_t *rank_out, int64_t *shape_out);

/* Canonicalises the layout, generates + compiles (hipRTC, gfx950) + caches the kernel for it.
 * Launches nothing; pointers are inspected for alignment and aliasing only.  Writes the
 * workspace size ewf_run will need for this layout (0 if none).  Needs a current HIP device. */
ewf_status ewf_plan(ewf_exec *e, const ewf_tensor *in, int32_t nin, const ewf_tensor *out,
                    int32_t nout, size_t *workspace_bytes);

/* Zero-fills a workspace with a fill kernel (asynchronous, on `stream`; safe to record into
 * a HIP graph).  Optional: the kernels write every workspace word before reading it, so a
 * workspace needs no initialisation; its contents after a run are unspecified.  Runs that may
 * overlap in time must not share a workspace. */
ewf_status ewf_workspace_init(void *workspace, size_t workspace_bytes, void *hip_stream);

/* Launches the planned kernel(s) on hip_stream (a hipStream_t; NULL = the null stream).
 * scalars: host array, one double per ewf_scalar in creation order (converted to the
 * scalar's type).  Plans implicitly if this layout has not been planned.
 * workspace may be NULL when the plan needs none. */
ewf_status ewf_run(ewf_exec *e, const ewf_tensor *in, int32_t nin, const double *scalars,
                   int32_t nscalars, const ewf_tensor *out, int32_t nout, void *workspace,
                   size_t workspace_bytes, void *hip_stream);

/* ewf_run for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results as ewf_run, but
 * the workspace is a static device array of EWF_STATIC_WORKSPACE_BYTES inside the library (each
 * GPU the library runs on holds it until the process ends), and the call sets nothing up: it
 * calls no hipMalloc, hipFree, compiler or module loader.  The layout must have been planned
 * before with ewf_plan while the same device was current (that compiles the kernels and loads
 * them); otherwise EWF_EINVAL.  A layout whose plan needs a larger workspace is EWF_ENOMEM: use
 * ewf_run with a workspace of your own.  Every call on one GPU shares that GPU's array: calls
 * that may overlap in time (different streams, threads or processes' worth of executables) race;
 * calls on one stream do not.  Nothing needs clearing between calls (see ewf_workspace_init). */
#define EWF_STATIC_WORKSPACE_BYTES (4u << 20)
ewf_status ewf_run_static(ewf_exec *e, const ewf_tensor *in, int32_t nin, const double *scalars,
                          int32_t nscalars, const ewf_tensor *out, int32_t nout, void *hip_stream);

/* The arguments of ewf_run gathered in one structure, for launch loops driven from another
 * language: a prepared call is passed as a single pointer (section 2.3, function execution:
 * with many operations on small operands the overhead of each call from the calling language is
 * what counts).  Same semantics and errors as ewf_run; the structure and everything it points
 * to are the caller's and may be changed between calls. */
typedef struct {
    ewf_exec *exec;
    const ewf_tensor *in;
    const ewf_tensor *out;
    const double *scalars;
    void *workspace;
    size_t workspace_bytes;
    void *hip_stream;
    int32_t nin, nout, nscalars, reserved;
} ewf_call;
ewf_status ewf_run_call(const ewf_call *call);
/* Runs `ncalls` prepared calls in order, each on its own hip_stream field -- the loop over the
 * steps of a prepared sequence runs inside the library, as the paper's C virtual machine runs
 * the loop over a function's nodes in C (section 2.3).  Stops at the first failing call,
 * returns its status and, when `failed` is not NULL, stores its index there. */
ewf_status ewf_run_sequence(const ewf_call *calls, int32_t ncalls, int32_t *failed);

const char *ewf_last_error(void);

/* ---- introspection, used by host-only tests and tools ---- */

typedef struct {
    int32_t kernel_class;     /* 0 none (empty), 1 tile element-wise, 2 tile + split reduce,
                                 3 row-resident reduce, 4 column reduce (kept axis fastest),
                                 5 several kernels (reductions materialised in the workspace;
                                 grid_blocks then counts the kernels' stages), 6 short rows,
                                 one thread per row                                          */
    int32_t rank;             /* canonical rank after dropping/merging dimensions            */
    int64_t extent[EWF_MAX_DIMS];
    int32_t reduced[EWF_MAX_DIMS];  /* 1 if the canonical dimension is reduced                */
    int32_t vec;              /* elements per memory access along the innermost dimension    */
    int32_t index_bits;       /* 32 or 64                                                    */
    int32_t noperands;        /* inputs then outputs                                         */
    int32_t block_threads;
    int32_t grid_blocks;
    int32_t lds_bytes;
    int32_t staged_operands;  /* number of operands staged through LDS                       */
    int64_t tile[EWF_MAX_DIMS];
} ewf_plan_info;

/* One node of a graph under construction, as the library holds it (lets a test read back what
 * ewf_grad appended). kind: 0 input, 1 scalar, 2 literal, 3 iota, 4 apply, 5 cast, 6 reduce. */
typedef struct {
    int32_t kind;
    int32_t op;               /* apply: ewf_op; reduce: ewf_redop; cast: target ewf_dtype      */
    int32_t nargs;
    int32_t args[3];
    int32_t index;            /* input / scalar ordinal; iota axis                            */
    uint32_t axes;            /* reduce: bit d set = axis d reduced                           */
    int32_t keep;             /* reduce: reduced axes stay in output shapes                   */
    int32_t vtype;            /* value type (EWF_F32 or EWF_I32)                              */
    int32_t storage;          /* input: storage type                                          */
    uint32_t bcast;           /* bit d set = constant along axis d                            */
    double cval;              /* literal                                                      */
} ewf_node_info;
int32_t ewf_debug_graph_count(const ewf_graph *g);
ewf_status ewf_debug_graph_node(const ewf_graph *g, int32_t i, ewf_node_info *info);

/* Describes the most recent plan made (or looked up) on this executable. */
ewf_status ewf_debug_plan_info(ewf_exec *e, ewf_plan_info *info);
/* Canonical element strides of operand k (inputs first, then outputs) of the last plan. */
ewf_status ewf_debug_operand_strides(ewf_exec *e, int32_t k, int64_t *strides_out);
/* Generated HIP source of the last plan (library-owned, valid until the next plan). */
const char *ewf_debug_source(ewf_exec *e);
/* A plan in several passes (kernel_class 5, grid_blocks = number of stages): the plan and the
 * generated source of stage `stage`, in execution order.  EWF_EINVAL when the last plan has no
 * such stage. */
ewf_status ewf_debug_stage_plan_info(ewf_exec *e, int32_t stage, ewf_plan_info *info);
const char *ewf_debug_stage_source(ewf_exec *e, int32_t stage);
/* Number of kernels compiled so far by this executable (cache misses). */
int32_t ewf_debug_compile_count(ewf_exec *e);
/* Nodes of the scalar graph as described, and after the rewrites of ewf_compile (section
 * 2.2.1 of the paper: canonicalisation merges duplicates and folds constants, stabilisation
 * replaces log(1 + x) by log1p(x)). */
ewf_status ewf_debug_graph_size(ewf_exec *e, int32_t *nodes_described, int32_t *nodes_compiled);

/* Process-wide counts of kernel sources served from memory, from the disk cache, and compiled. */
ewf_status ewf_debug_cache_stats(int32_t *memory_hits, int32_t *disk_hits, int32_t *compiles);

/* The most run-time compilations that were in progress at the same moment so far in this process
 * (distinct kernel sources are compiled concurrently; a second request for a source that is
 * being compiled waits for the first). */
ewf_status ewf_debug_peak_concurrent_compiles(int32_t *peak);
/* Test hook for the rule that no C++ exception crosses this boundary: arms a fault on the calling
 * thread.  The library passes fault points where it asks for host memory (adding a graph node,
 * looking a plan up or making one); after `after` further points the next one throws --
 * kind 1 as running out of memory (the call then returns EWF_ENOMEM), kind 2 as any other
 * exception (EWF_EINVAL, its text in ewf_last_error); kind 0 disarms.  A fault fires once. */
ewf_status ewf_debug_inject_fault(int32_t kind, int32_t after);

/* ---- measurement aid ---- */

/* Times the main kernel of the following ewf_run calls on this executable (the streaming pass;
 * not the small second kernel that folds partial results; every stage of a plan in several
 * passes): each such launch gets a pair of HIP events tied to that dispatch alone, so the
 * durations are the kernel's own, as a profiler's kernel trace reports them, without the cost
 * of recording events around a launch call.  `slots` = number of kernel launches to record
 * (events are created here, none by ewf_run); 0 turns timing off. */
ewf_status ewf_debug_time_kernels(ewf_exec *e, int32_t slots);
/* Waits for the recorded launches and writes their durations in milliseconds, in launch order;
 * *count = how many were written.  Recording starts again from the first slot. */
ewf_status ewf_debug_kernel_times(ewf_exec *e, float *ms, int32_t capacity, int32_t *count);

/* Plain device-to-device copy of nbytes (multiple of 16, 16-byte aligned pointers) with the
 * library's own dwordx4 grid-stride kernel: the measured ceiling that bandwidth figures and
 * hardware-counter scale factors are quoted against. */
ewf_status ewf_copy_bytes(void *dst, const void *src, size_t nbytes, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* EWF_H */
