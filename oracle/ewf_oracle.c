/*
 * ewf_oracle.c -- reference evaluator for fused element-wise + reduce expressions.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must compute; it is
 * slow on purpose and shares no code, header, table or helper with the GPU library.  Only
 * the tests, the smoke check and the benchmark's CPU-baseline leg may load it.
 *
 * What it computes (paper section 2.1.1 for the graph and the broadcastable pattern,
 * section 2.2.1 "Specialize" for fusion, "Inplace" for strided views):
 *
 *   A fused element-wise computation is, by definition, the point-wise application of a
 *   directed acyclic graph of scalar operations.  Fusing the loops does not change the
 *   value, so the oracle is that definition written out: for every output coordinate,
 *   read each operand at that coordinate (index forced to 0 on the dimensions the
 *   operand's type flags as broadcastable, address = base + sum_d index_d * stride_d),
 *   evaluate the scalar graph in static-single-assignment order, store.
 *
 *   A reduce node folds its argument over the listed axes.  Every value carries the shape
 *   "full extent where it varies, 1 where it is broadcastable"; the reduction runs over
 *   the argument's own extent on each reduced axis, sequentially in row-major order.
 *   Reduce nodes are materialised one after the other in graph order into double buffers,
 *   so later nodes (for instance exp(x - rowmax)) read them like broadcast operands.
 *
 * Arithmetic: every real-valued scalar operation is evaluated in IEEE double with <math.h>;
 * operands are widened exactly from their storage type; explicit cast nodes round
 * (to float32 / float16 with round-to-nearest-even, to int32 by truncation with saturation);
 * each output is rounded once to its storage type.  Integer-valued nodes use 32-bit
 * two's-complement arithmetic.  Reductions accumulate in double.
 *
 * Pins: every operation, the broadcast rule, the stride rule, reductions, argmax ties and
 * the float16 conversions are checked in tests/test_oracle_*.py against printed closed
 * forms, hand-computed tensors, identities and independent numpy float64 expressions.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define ORC_MAXD 8
#define ORC_MAXNODES 256

/* node kinds */
enum { K_INPUT = 0, K_SCALAR = 1, K_CONST = 2, K_IOTA = 3, K_APPLY = 4, K_CAST = 5, K_REDUCE = 6 };
/* value types */
enum { T_REAL = 0, T_INT = 1 };
/* storage types */
enum { S_F32 = 0, S_F16 = 1, S_I32 = 2 };
/* scalar operations (numbering private to the oracle) */
enum {
    O_ADD = 0, O_SUB, O_MUL, O_DIV, O_NEG, O_ABS, O_EXP, O_LOG, O_LOG1P, O_SQRT, O_TANH,
    O_SIGMOID, O_MAX, O_MIN, O_POW, O_WHERE, O_GT, O_GE, O_LT, O_LE, O_EQ, O_NE, O_EXPM1,
    O_SQR, O_RECIP, O_NOPS
};
/* reductions */
enum { R_SUM = 0, R_MAX, R_MIN, R_PROD, R_ARGMAX };

/* error codes */
enum {
    ORC_OK = 0, ORC_EINVAL = -1, ORC_ETYPE = -2, ORC_ESHAPE = -3, ORC_ENOMEM = -4
};

typedef struct {
    int32_t kind;
    int32_t op;       /* K_APPLY: operation; K_REDUCE: reduction; K_CAST: target storage type;
                         K_SCALAR / K_CONST: value type */
    int32_t nargs;
    int32_t args[3];
    int32_t index;    /* K_INPUT: input number; K_SCALAR: scalar number; K_IOTA: axis */
    uint32_t axes;    /* K_REDUCE: bit d set = axis d is reduced */
    double cval;      /* K_CONST */
} orc_node;

typedef struct {
    void *data;
    int32_t storage;
    uint32_t bcast;           /* bit d set = dimension d is flagged broadcastable (extent 1) */
    int64_t shape[ORC_MAXD];
    int64_t strides[ORC_MAXD]; /* in elements */
} orc_tensor;

/* ---------------------------------------------------------------- float16 <-> double */

/* IEEE binary16 bits -> double (exact). */
static double half_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, e = (h >> 10) & 0x1f, m = h & 0x3ff;
    double v;
    if (e == 0)
        v = ldexp((double)m, -24);                 /* zero and subnormals: m * 2^-24 */
    else if (e == 31)
        v = m ? NAN : INFINITY;
    else
        v = ldexp((double)(m + 1024), e - 25);     /* (1 + m/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* double -> IEEE binary16 bits, round to nearest, ties to even, overflow to infinity. */
static uint16_t double_to_half(double x)
{
    uint16_t sign = signbit(x) ? 0x8000u : 0;
    double a = fabs(x);
    if (isnan(x)) return (uint16_t)(sign | 0x7e00u);
    if (isinf(a)) return (uint16_t)(sign | 0x7c00u);
    if (a == 0.0) return sign;
    int ex;
    (void)frexp(a, &ex);              /* a = f * 2^ex, f in [0.5,1) ; so a in [2^(ex-1), 2^ex) */
    int e = ex - 1;                   /* unbiased exponent of the leading bit */
    if (e < -14) e = -14;             /* subnormal range shares the quantum 2^-24 */
    /* quantum of the target format at this exponent: 2^(e-10) */
    double q = ldexp(a, 10 - e);      /* a in units of the quantum: in [1024,2048) if normal */
    double fl = floor(q);
    double rem = q - fl;
    if (rem > 0.5 || (rem == 0.5 && fmod(fl, 2.0) == 1.0)) fl += 1.0;
    /* fl is now an integer in [0, 2048] */
    if (fl >= 2048.0) { fl = 1024.0; e += 1; }
    if (e > 15) return (uint16_t)(sign | 0x7c00u);
    uint32_t mant = (uint32_t)fl;
    if (mant < 1024u)                 /* subnormal (only possible when e == -14) */
        return (uint16_t)(sign | mant);
    return (uint16_t)(sign | ((uint32_t)(e + 15) << 10) | (mant - 1024u));
}

/* ---------------------------------------------------------------- analysis */

typedef struct {
    int ndim, nnodes, nin, nscal;
    const orc_node *nodes;
    const orc_tensor *in;
    const double *scal;
    int64_t full[ORC_MAXD];
    int vtype[ORC_MAXNODES];        /* T_REAL / T_INT */
    uint32_t vbc[ORC_MAXNODES];     /* bit d set = value does not vary along d */
    double *rbuf[ORC_MAXNODES];     /* materialised reduce results */
} orc_ctx;

static int wrap32(int64_t v) { return (int32_t)(uint32_t)(uint64_t)v; }

static int analyse(orc_ctx *c)
{
    const uint32_t all = (c->ndim >= 32) ? 0xffffffffu : ((1u << c->ndim) - 1u);
    for (int n = 0; n < c->nnodes; n++) {
        const orc_node *nd = &c->nodes[n];
        for (int a = 0; a < nd->nargs; a++)
            if (nd->args[a] < 0 || nd->args[a] >= n) return ORC_EINVAL;
        switch (nd->kind) {
        case K_INPUT:
            if (nd->index < 0 || nd->index >= c->nin) return ORC_EINVAL;
            c->vtype[n] = (c->in[nd->index].storage == S_I32) ? T_INT : T_REAL;
            c->vbc[n] = c->in[nd->index].bcast & all;
            break;
        case K_SCALAR:
            if (nd->index < 0 || nd->index >= c->nscal) return ORC_EINVAL;
            c->vtype[n] = nd->op; c->vbc[n] = all;
            break;
        case K_CONST:
            c->vtype[n] = nd->op; c->vbc[n] = all;
            break;
        case K_IOTA:
            if (nd->index < 0 || nd->index >= c->ndim) return ORC_EINVAL;
            c->vtype[n] = T_INT; c->vbc[n] = all & ~(1u << nd->index);
            break;
        case K_CAST:
            if (nd->nargs != 1) return ORC_EINVAL;
            c->vtype[n] = (nd->op == S_I32) ? T_INT : T_REAL;
            c->vbc[n] = c->vbc[nd->args[0]];
            break;
        case K_REDUCE: {
            if (nd->nargs != 1) return ORC_EINVAL;
            if (nd->axes == 0 || (nd->axes & ~all)) return ORC_EINVAL;
            c->vtype[n] = (nd->op == R_ARGMAX) ? T_INT : c->vtype[nd->args[0]];
            c->vbc[n] = c->vbc[nd->args[0]] | nd->axes;
            break;
        }
        case K_APPLY: {
            int t0 = nd->nargs > 0 ? c->vtype[nd->args[0]] : T_REAL;
            uint32_t bc = all;
            for (int a = 0; a < nd->nargs; a++) bc &= c->vbc[nd->args[a]];
            c->vbc[n] = bc;
            switch (nd->op) {
            case O_ADD: case O_SUB: case O_MUL: case O_MAX: case O_MIN:
                if (nd->nargs != 2 || c->vtype[nd->args[1]] != t0) return ORC_ETYPE;
                c->vtype[n] = t0; break;
            case O_NEG: case O_ABS: case O_SQR:
                if (nd->nargs != 1) return ORC_ETYPE;
                c->vtype[n] = t0; break;
            case O_DIV: case O_POW:
                if (nd->nargs != 2 || t0 != T_REAL || c->vtype[nd->args[1]] != T_REAL) return ORC_ETYPE;
                c->vtype[n] = T_REAL; break;
            case O_EXP: case O_LOG: case O_LOG1P: case O_SQRT: case O_TANH: case O_SIGMOID:
            case O_EXPM1: case O_RECIP:
                if (nd->nargs != 1 || t0 != T_REAL) return ORC_ETYPE;
                c->vtype[n] = T_REAL; break;
            case O_GT: case O_GE: case O_LT: case O_LE: case O_EQ: case O_NE:
                if (nd->nargs != 2 || c->vtype[nd->args[1]] != t0) return ORC_ETYPE;
                c->vtype[n] = T_INT; break;
            case O_WHERE:
                if (nd->nargs != 3 || c->vtype[nd->args[1]] != c->vtype[nd->args[2]]) return ORC_ETYPE;
                c->vtype[n] = c->vtype[nd->args[1]]; break;
            default: return ORC_EINVAL;
            }
            break;
        }
        default: return ORC_EINVAL;
        }
    }
    return ORC_OK;
}

/* Mark the nodes that must be evaluated per element to obtain `target`.  Reduce nodes are
 * leaves here: their value is read from the buffer filled earlier. */
static void mark_needed(const orc_ctx *c, int target, unsigned char *need)
{
    memset(need, 0, (size_t)c->nnodes);
    need[target] = 1;
    for (int n = target; n >= 0; n--) {
        if (!need[n]) continue;
        const orc_node *nd = &c->nodes[n];
        if (nd->kind == K_REDUCE && n != target) continue;
        if (nd->kind == K_REDUCE) continue;
        for (int a = 0; a < nd->nargs; a++) need[nd->args[a]] = 1;
    }
}

/* Row-major offset into the buffer of a reduce node: its shape is the full extent on the
 * dimensions where it varies and 1 elsewhere. */
static int64_t rbuf_offset(const orc_ctx *c, int n, const int64_t *coord)
{
    int64_t off = 0;
    for (int d = 0; d < c->ndim; d++) {
        if (c->vbc[n] & (1u << d)) continue;
        off = off * c->full[d] + coord[d];
    }
    return off;
}

static double load_elem(const orc_tensor *t, int ndim, const int64_t *coord)
{
    int64_t off = 0;
    for (int d = 0; d < ndim; d++) {
        int64_t i = (t->bcast & (1u << d)) ? 0 : coord[d];
        off += i * t->strides[d];
    }
    switch (t->storage) {
    case S_F32: return (double)((const float *)t->data)[off];
    case S_F16: return half_to_double(((const uint16_t *)t->data)[off]);
    default:    return (double)((const int32_t *)t->data)[off];
    }
}

static double sigmoid_d(double x)
{
    /* 1/(1+e^-x); the mirrored form avoids overflow of e^-x for very negative x */
    if (x >= 0.0) return 1.0 / (1.0 + exp(-x));
    double e = exp(x);
    return e / (1.0 + e);
}

static double apply_real(int op, const double *v)
{
    switch (op) {
    case O_ADD: return v[0] + v[1];
    case O_SUB: return v[0] - v[1];
    case O_MUL: return v[0] * v[1];
    case O_DIV: return v[0] / v[1];
    case O_NEG: return -v[0];
    case O_ABS: return fabs(v[0]);
    case O_EXP: return exp(v[0]);
    case O_LOG: return log(v[0]);
    case O_LOG1P: return log1p(v[0]);
    case O_SQRT: return sqrt(v[0]);
    case O_TANH: return tanh(v[0]);
    case O_SIGMOID: return sigmoid_d(v[0]);
    case O_MAX: return (isnan(v[0]) || isnan(v[1])) ? NAN : (v[0] > v[1] ? v[0] : v[1]);
    case O_MIN: return (isnan(v[0]) || isnan(v[1])) ? NAN : (v[0] < v[1] ? v[0] : v[1]);
    case O_POW: return pow(v[0], v[1]);
    case O_EXPM1: return expm1(v[0]);
    case O_SQR: return v[0] * v[0];
    case O_RECIP: return 1.0 / v[0];
    default: return NAN;
    }
}

static double apply_int(int op, const double *v)
{
    int64_t a = (int64_t)v[0], b = (int64_t)v[1];
    switch (op) {
    case O_ADD: return (double)wrap32(a + b);
    case O_SUB: return (double)wrap32(a - b);
    case O_MUL: return (double)wrap32(a * b);
    case O_NEG: return (double)wrap32(-a);
    case O_ABS: return (double)wrap32(a < 0 ? -a : a);
    case O_SQR: return (double)wrap32(a * a);
    case O_MAX: return (double)(a > b ? a : b);
    case O_MIN: return (double)(a < b ? a : b);
    default: return 0.0;
    }
}

static double cast_value(int target, int from_type, double v)
{
    switch (target) {
    case S_F32: return (double)(float)v;                 /* int32 -> f32 and f64 -> f32: RNE */
    case S_F16: return half_to_double(double_to_half(v));
    default:                                             /* to int32 */
        if (from_type == T_INT) return v;
        if (isnan(v)) return 0.0;
        if (v >= 2147483647.0) return 2147483647.0;
        if (v <= -2147483648.0) return -2147483648.0;
        return trunc(v);
    }
}

/* Evaluate, at one coordinate, every node flagged in `need`, in graph order. */
static void eval_at(const orc_ctx *c, const unsigned char *need, int upto, const int64_t *coord,
                    double *val)
{
    for (int n = 0; n <= upto; n++) {
        if (!need[n]) continue;
        const orc_node *nd = &c->nodes[n];
        switch (nd->kind) {
        case K_INPUT: val[n] = load_elem(&c->in[nd->index], c->ndim, coord); break;
        case K_SCALAR:
            val[n] = (nd->op == T_INT) ? (double)wrap32((int64_t)c->scal[nd->index])
                                       : (double)(float)c->scal[nd->index];
            break;
        case K_CONST:
            /* a literal has a type like any other value: float32 or int32 */
            val[n] = (nd->op == T_INT) ? (double)wrap32((int64_t)nd->cval) : (double)(float)nd->cval;
            break;
        case K_IOTA: val[n] = (double)coord[nd->index]; break;
        case K_CAST: val[n] = cast_value(nd->op, c->vtype[nd->args[0]], val[nd->args[0]]); break;
        case K_REDUCE: val[n] = c->rbuf[n][rbuf_offset(c, n, coord)]; break;
        case K_APPLY: {
            double v[3] = {0, 0, 0};
            for (int a = 0; a < nd->nargs; a++) v[a] = val[nd->args[a]];
            int at = c->vtype[nd->args[0]];
            switch (nd->op) {
            case O_WHERE: val[n] = (v[0] != 0.0) ? v[1] : v[2]; break;  /* NaN != 0 is true */
            case O_GT: val[n] = v[0] > v[1]; break;
            case O_GE: val[n] = v[0] >= v[1]; break;
            case O_LT: val[n] = v[0] < v[1]; break;
            case O_LE: val[n] = v[0] <= v[1]; break;
            case O_EQ: val[n] = v[0] == v[1]; break;
            case O_NE: val[n] = v[0] != v[1]; break;
            default: val[n] = (at == T_INT) ? apply_int(nd->op, v) : apply_real(nd->op, v);
            }
            break;
        }
        }
    }
}

/* Extent of value n along d. */
static int64_t vext(const orc_ctx *c, int n, int d)
{
    return (c->vbc[n] & (1u << d)) ? 1 : c->full[d];
}

static int materialise_reduce(orc_ctx *c, int n, int nthreads)
{
    const orc_node *nd = &c->nodes[n];
    const int arg = nd->args[0];
    const int is_int = (c->vtype[arg] == T_INT);
    int64_t nkeep = 1, nred = 1;
    int kd[ORC_MAXD], nk = 0, rd[ORC_MAXD], nr = 0;
    for (int d = 0; d < c->ndim; d++) {
        if (nd->axes & (1u << d)) { rd[nr++] = d; nred *= vext(c, arg, d); }
        else if (!(c->vbc[n] & (1u << d))) { kd[nk++] = d; nkeep *= c->full[d]; }
    }
    if (nred == 0 && (nd->op == R_MAX || nd->op == R_MIN || nd->op == R_ARGMAX)) return ORC_ESHAPE;
    c->rbuf[n] = (double *)malloc(sizeof(double) * (size_t)(nkeep > 0 ? nkeep : 1));
    if (!c->rbuf[n]) return ORC_ENOMEM;
    unsigned char need[ORC_MAXNODES];
    mark_needed(c, arg, need);

#pragma omp parallel for num_threads(nthreads) schedule(static) if (nthreads > 1)
    for (int64_t k = 0; k < nkeep; k++) {
        int64_t coord[ORC_MAXD] = {0};
        double val[ORC_MAXNODES];
        int64_t rem = k;
        for (int j = nk - 1; j >= 0; j--) { coord[kd[j]] = rem % c->full[kd[j]]; rem /= c->full[kd[j]]; }
        double acc = 0.0;
        int64_t best = 0;
        switch (nd->op) {
        case R_SUM: acc = 0.0; break;
        case R_PROD: acc = 1.0; break;
        default: break;
        }
        for (int64_t r = 0; r < nred; r++) {
            int64_t rr = r;
            for (int j = nr - 1; j >= 0; j--) {
                int64_t e = vext(c, arg, rd[j]);
                coord[rd[j]] = rr % e; rr /= e;
            }
            eval_at(c, need, arg, coord, val);
            double v = val[arg];
            switch (nd->op) {
            case R_SUM: acc = is_int ? (double)wrap32((int64_t)acc + (int64_t)v) : acc + v; break;
            case R_PROD: acc = is_int ? (double)wrap32((int64_t)acc * (int64_t)v) : acc * v; break;
            case R_MAX:
                if (r == 0) acc = v;
                else if (!isnan(acc) && (isnan(v) || v > acc)) acc = v;
                break;
            case R_MIN:
                if (r == 0) acc = v;
                else if (!isnan(acc) && (isnan(v) || v < acc)) acc = v;
                break;
            case R_ARGMAX:                      /* first occurrence of the maximum: its position in the
                                                   row-major order of the reduced axes (r walks them in
                                                   that order; with one axis it is the coordinate) */
                if (r == 0) { acc = v; best = 0; }
                else if (!isnan(acc) && (isnan(v) || v > acc)) { acc = v; best = r; }
                break;
            }
        }
        c->rbuf[n][k] = (nd->op == R_ARGMAX) ? (double)best : acc;
    }
    return ORC_OK;
}

static int write_output(orc_ctx *c, int n, const orc_tensor *out, int nthreads)
{
    /* the output tensor has rank ndim: extent 1 where the value is broadcastable */
    int64_t total = 1;
    for (int d = 0; d < c->ndim; d++) {
        if (out->shape[d] != vext(c, n, d)) return ORC_ESHAPE;
        total *= out->shape[d];
    }
    if (c->vtype[n] == T_INT && out->storage != S_I32) return ORC_ETYPE;
    if (c->vtype[n] == T_REAL && out->storage == S_I32) return ORC_ETYPE;
    unsigned char need[ORC_MAXNODES];
    mark_needed(c, n, need);
    if (c->nodes[n].kind == K_REDUCE) need[n] = 1;
    int64_t outer = (c->ndim > 0) ? out->shape[0] : 1;
    int64_t inner = (outer > 0) ? total / outer : 0;

#pragma omp parallel for num_threads(nthreads) schedule(static) if (nthreads > 1)
    for (int64_t o = 0; o < outer; o++) {
        double val[ORC_MAXNODES];
        int64_t coord[ORC_MAXD] = {0};
        for (int64_t q = 0; q < inner; q++) {
            int64_t rem = q;
            for (int d = c->ndim - 1; d >= 1; d--) { coord[d] = rem % out->shape[d]; rem /= out->shape[d]; }
            if (c->ndim > 0) coord[0] = o;
            eval_at(c, need, n, coord, val);
            int64_t off = 0;
            for (int d = 0; d < c->ndim; d++) off += coord[d] * out->strides[d];
            switch (out->storage) {
            case S_F32: ((float *)out->data)[off] = (float)val[n]; break;
            case S_F16: ((uint16_t *)out->data)[off] = double_to_half(val[n]); break;
            default:    ((int32_t *)out->data)[off] = (int32_t)val[n]; break;
            }
        }
    }
    return ORC_OK;
}

/*
 * Evaluate a graph.
 *   ndim        rank shared by every operand and value
 *   full        iteration-space extents (what a non-broadcastable dimension must measure)
 *   nodes       graph in static-single-assignment order (arguments refer to earlier nodes)
 *   in          input tensors, rank ndim; a flagged dimension must have extent 1
 *   scal        run-time scalars
 *   out_nodes   node computed by each output; outs[k] has rank ndim with extent 1 on the
 *               dimensions where that node is broadcastable
 * Returns 0 or a negative ORC_E* code.  Host memory only.
 */
int orc_eval(int ndim, const int64_t *full, const orc_node *nodes, int nnodes,
             const orc_tensor *in, int nin, const double *scal, int nscal,
             const int32_t *out_nodes, const orc_tensor *outs, int nout, int nthreads)
{
    if (ndim < 0 || ndim > ORC_MAXD || nnodes <= 0 || nnodes > ORC_MAXNODES) return ORC_EINVAL;
    orc_ctx c;
    memset(&c, 0, sizeof c);
    c.ndim = ndim; c.nnodes = nnodes; c.nin = nin; c.nscal = nscal;
    c.nodes = nodes; c.in = in; c.scal = scal;
    for (int d = 0; d < ndim; d++) c.full[d] = full[d];
    int rc = analyse(&c);
    if (rc) return rc;
    /* the broadcastable pattern is a guarantee: flagged => extent 1, unflagged => full extent */
    for (int k = 0; k < nin; k++)
        for (int d = 0; d < ndim; d++) {
            int64_t want = (in[k].bcast & (1u << d)) ? 1 : full[d];
            if (in[k].shape[d] != want) return ORC_ESHAPE;
        }
    if (nthreads < 1) nthreads = 1;
    for (int n = 0; n < nnodes && rc == ORC_OK; n++)
        if (nodes[n].kind == K_REDUCE) rc = materialise_reduce(&c, n, nthreads);
    for (int k = 0; k < nout && rc == ORC_OK; k++) {
        if (out_nodes[k] < 0 || out_nodes[k] >= nnodes) { rc = ORC_EINVAL; break; }
        rc = write_output(&c, out_nodes[k], &outs[k], nthreads);
    }
    for (int n = 0; n < nnodes; n++) free(c.rbuf[n]);
    return rc;
}

/* Conversions exported so the tests can pin them against an independent implementation. */
uint16_t orc_double_to_half(double x) { return double_to_half(x); }
double orc_half_to_double(uint16_t h) { return half_to_double(h); }
