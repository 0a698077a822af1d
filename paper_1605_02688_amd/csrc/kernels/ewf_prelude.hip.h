// Device-side helpers shared by every generated kernel (gfx950, wave64).
//
// This text is compiled at run time, in front of the per-expression code the generator
// emits.  It holds: wide aligned memory accesses, storage <-> value conversions, the scalar
// operations in an accurate float32 flavour and a native-rate flavour, and the wavefront /
// workgroup reduction used by the fused reduce kernels (cross-lane DPP inside a row of 16
// lanes, lane permutes across rows, LDS across wavefronts).  Results that span workgroups
// are exchanged through the workspace and folded by a second kernel: on this chip an
// agent-scope fence writes back and invalidates a whole L2 slice, and contended global
// atomics cost a memory round trip each, so the kernels use neither.
#ifndef EWF_PRELUDE_H
#define EWF_PRELUDE_H

typedef _Float16 ewf_half;
typedef unsigned int ewf_u32;

#define EWF_DEV __device__ __forceinline__

// ------------------------------------------------------------------ wide memory accesses

template <int B> struct ewf_align { static constexpr int value = B >= 16 ? 16 : B; };

template <typename T, int N>
struct alignas(ewf_align<N * (int)sizeof(T)>::value) ewf_vec {
    T e[N];
};

// float16 vectors of two or more elements are also visible as the 32-bit words that hold
// pairs of halves, so that unpacking can work on whole registers
#define EWF_HALF_VEC(N)                                        \
    template <>                                                \
    struct alignas(ewf_align<N * 2>::value) ewf_vec<ewf_half, N> { \
        union {                                                \
            ewf_half e[N];                                     \
            unsigned w[N / 2];                                 \
        };                                                     \
    };
EWF_HALF_VEC(2)
EWF_HALF_VEC(4)
EWF_HALF_VEC(8)
EWF_HALF_VEC(16)
#undef EWF_HALF_VEC

// One aligned access of N elements (N * sizeof(T) bytes, in 16-byte pieces when larger).
template <typename T, int N>
EWF_DEV ewf_vec<T, N> ewf_ld(const T *p)
{
    return *reinterpret_cast<const ewf_vec<T, N> *>(p);
}

template <typename T, int N>
EWF_DEV void ewf_st(T *p, const ewf_vec<T, N> &v)
{
    *reinterpret_cast<ewf_vec<T, N> *>(p) = v;
}

// The same accesses for addresses that are aligned to the element only (rows with an odd pitch,
// views that start inside a vector).  The memory instructions of this target take any address;
// declaring the reduced alignment keeps the compiler from assuming more.
template <typename T, int N>
struct __attribute__((packed, aligned(sizeof(T)))) ewf_vec_u { ewf_vec<T, N> v; };

template <typename T, int N>
EWF_DEV ewf_vec<T, N> ewf_ld_u(const T *p)
{
    return reinterpret_cast<const ewf_vec_u<T, N> *>(p)->v;
}

template <typename T, int N>
EWF_DEV void ewf_st_u(T *p, const ewf_vec<T, N> &v)
{
    reinterpret_cast<ewf_vec_u<T, N> *>(p)->v = v;
}

// A value at an address that is the same in every lane and that no lane of this launch writes
// before reading it: read through the scalar unit (one request per wavefront, its own wait
// counter, the result in a scalar register).
template <typename T>
EWF_DEV T ewf_ld_uniform(const T *p)
{
    return *(const __attribute__((address_space(4))) T *)p;
}

// Streaming flavour of the same accesses for operands that are touched exactly once and
// are much larger than the caches: the non-temporal hint keeps them from displacing the
// broadcast operands and measurably raises sustained HBM throughput.
typedef unsigned int ewf_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int ewf_u32x2 __attribute__((ext_vector_type(2)));

template <typename T, int N>
EWF_DEV ewf_vec<T, N> ewf_ld_nt(const T *p)
{
    constexpr int B = N * (int)sizeof(T);
    ewf_vec<T, N> r;
    if constexpr (B % 16 == 0) {
        const ewf_u32x4 *s = reinterpret_cast<const ewf_u32x4 *>(p);
        ewf_u32x4 *d = reinterpret_cast<ewf_u32x4 *>(&r);
#pragma unroll
        for (int i = 0; i < B / 16; i++) d[i] = __builtin_nontemporal_load(s + i);
    } else if constexpr (B == 8) {
        *reinterpret_cast<ewf_u32x2 *>(&r) = __builtin_nontemporal_load(reinterpret_cast<const ewf_u32x2 *>(p));
    } else if constexpr (B == 4) {
        *reinterpret_cast<unsigned int *>(&r) = __builtin_nontemporal_load(reinterpret_cast<const unsigned int *>(p));
    } else {
        *reinterpret_cast<unsigned short *>(&r) = __builtin_nontemporal_load(reinterpret_cast<const unsigned short *>(p));
    }
    return r;
}

template <typename T, int N>
EWF_DEV void ewf_st_nt(T *p, const ewf_vec<T, N> &v)
{
    constexpr int B = N * (int)sizeof(T);
    if constexpr (B % 16 == 0) {
        ewf_u32x4 *d = reinterpret_cast<ewf_u32x4 *>(p);
        const ewf_u32x4 *s = reinterpret_cast<const ewf_u32x4 *>(&v);
#pragma unroll
        for (int i = 0; i < B / 16; i++) __builtin_nontemporal_store(s[i], d + i);
    } else if constexpr (B == 8) {
        __builtin_nontemporal_store(*reinterpret_cast<const ewf_u32x2 *>(&v), reinterpret_cast<ewf_u32x2 *>(p));
    } else if constexpr (B == 4) {
        __builtin_nontemporal_store(*reinterpret_cast<const unsigned int *>(&v), reinterpret_cast<unsigned int *>(p));
    } else {
        __builtin_nontemporal_store(*reinterpret_cast<const unsigned short *>(&v), reinterpret_cast<unsigned short *>(p));
    }
}

// ------------------------------------------------------------------ storage <-> value

EWF_DEV float ewf_in(float x) { return x; }
EWF_DEV float ewf_in(ewf_half x) { return (float)x; }
EWF_DEV int ewf_in(int x) { return x; }

// Element e of a float16 vector as float32.  Two halves share a register: the low one is
// converted in place; the high one goes through a mixed-precision multiply-add that selects
// the high half by itself (x * 1 + 0, exact), which saves the shift a plain conversion needs.
template <int N>
EWF_DEV float ewf_in_h(const ewf_vec<ewf_half, N> &v, int e)
{
    if constexpr (N >= 2) {
        const unsigned w = v.w[e >> 1];
        if (e & 1) {
            float r;
            asm("v_fma_mix_f32 %0, %1, 1.0, 0 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w));
            return r;
        }
        return (float)__builtin_bit_cast(ewf_half, (unsigned short)w);
    } else {
        return (float)v.e[e];
    }
}

EWF_DEV float ewf_out_f32(float x) { return x; }
EWF_DEV ewf_half ewf_out_f16(float x) { return (ewf_half)x; }   // round to nearest even
EWF_DEV int ewf_out_i32(int x) { return x; }

EWF_DEV float ewf_round_f16(float x) { return (float)(ewf_half)x; }
EWF_DEV int ewf_f2i(float x)
{
    // truncation toward zero, saturating, NaN -> 0
    if (!(x == x)) return 0;
    if (x >= 2147483648.0f) return 2147483647;
    if (x <= -2147483648.0f) return (-2147483647 - 1);
    return (int)x;
}

EWF_DEV float ewf_bits_f32(ewf_u32 b) { return __uint_as_float(b); }

// ------------------------------------------------------------------ scalar operations

// max / min propagate NaN from either operand
EWF_DEV float ewf_max(float a, float b) { return ((a > b) | (a != a)) ? a : b; }
EWF_DEV float ewf_min(float a, float b) { return ((a < b) | (a != a)) ? a : b; }
EWF_DEV int ewf_max(int a, int b) { return a > b ? a : b; }
EWF_DEV int ewf_min(int a, int b) { return a < b ? a : b; }
EWF_DEV float ewf_abs(float a) { return fabsf(a); }
EWF_DEV int ewf_abs(int a) { return a < 0 ? (int)(0u - (ewf_u32)a) : a; }
EWF_DEV int ewf_addi(int a, int b) { return (int)((ewf_u32)a + (ewf_u32)b); }
EWF_DEV int ewf_subi(int a, int b) { return (int)((ewf_u32)a - (ewf_u32)b); }
EWF_DEV int ewf_muli(int a, int b) { return (int)((ewf_u32)a * (ewf_u32)b); }
EWF_DEV int ewf_negi(int a) { return (int)(0u - (ewf_u32)a); }

// where(c, a, b): a when c != 0; a NaN condition is "not equal to zero"
EWF_DEV bool ewf_truth(float c) { return c != 0.0f; }
EWF_DEV bool ewf_truth(int c) { return c != 0; }

// accurate float32 flavour (one to two units in the last place; tanh up to about six near |x| = 0.25)
struct ewf_acc {
    // exp(x) = 2^(x * log2 e).  The product is formed in two pieces: its float32 rounding t,
    // and r = the rounding error of t plus x times the part of log2 e that float32 drops.
    // The hardware exp2 (one unit in the last place over the whole range, no argument
    // reduction needed) takes t, and r corrects the result to first order: 2^r = 1 + r ln 2
    // for |r| < 2^-16.  Seven instructions instead of the library routine's fifteen or so.
    // Infinite x makes r NaN, and a finite x whose product overflows makes it infinite; the
    // median with 0.5 and 2 drops both (the hardware median returns the smallest number when an
    // operand is NaN) so that the result is the 0 or inf of exp2, while a NaN x still reaches the
    // result through t.  Results below the smallest normal number flush to zero.
    static EWF_DEV float exp(float x)
    {
        const float t = x * 1.44269502162933349609375f;                 // log2 e rounded
        float r = __builtin_fmaf(x, 1.44269502162933349609375f, -t);
        r = __builtin_fmaf(x, 1.92596298909109e-8f, r);                 // log2 e - rounded
        const float f = __builtin_amdgcn_fmed3f(__builtin_fmaf(r, 0.693147182464599609375f, 1.0f), 0.5f, 2.0f);
        return __builtin_amdgcn_exp2f(t) * f;
    }
    static EWF_DEV float log(float x) { return logf(x); }
    static EWF_DEV float log1p(float x) { return log1pf(x); }
    static EWF_DEV float expm1(float x) { return expm1f(x); }
    static EWF_DEV float sqrt(float x) { return sqrtf(x); }
    // 1 / y for y >= 1 (finite): the hardware reciprocal refined by one Newton step
    static EWF_DEV float recip_ge1(float y)
    {
        const float r = __builtin_amdgcn_rcpf(y);
        return __builtin_fmaf(__builtin_fmaf(-y, r, 1.0f), r, r);
    }
    // tanh: below 0.25 the odd series up to x^11 (relative error under one unit in the last
    // place); above, 1 - 2 / (exp(2|x|) + 1), whose subtraction amplifies the quotient's error at
    // most threefold there (about six units in the last place at the seam, one far from it).
    // The argument of exp is capped so that it stays finite (a NaN passes the comparison).
    static EWF_DEV float tanh(float x)
    {
        float a = fabsf(x);
        const float x2 = x * x;
        float p = __builtin_fmaf(x2, -0.00886323552990219656f, 0.02186948853615520282f);    // -1382/155925, 62/2835
        p = __builtin_fmaf(x2, p, -0.05396825396825396825f);                                // -17/315
        p = __builtin_fmaf(x2, p, 0.13333333333333333333f);                                 // 2/15
        p = __builtin_fmaf(x2, p, -0.33333333333333333333f);
        p = __builtin_fmaf(x2 * a, p, a);
        const float c = (a > 44.0f) ? 44.0f : a;
        const float e = exp(c + c);
        const float t = __builtin_fmaf(-2.0f, recip_ge1(e + 1.0f), 1.0f);
        return copysignf((a < 0.25f) ? p : t, x);
    }
    // sigmoid: 1 / (1 + exp(-x)) with the argument of exp capped at 88 (the result is then below
    // the smallest normal number and comes out as 0 or a subnormal)
    static EWF_DEV float sigmoid(float x)
    {
        const float m = -x;
        return recip_ge1(1.0f + exp((m > 88.0f) ? 88.0f : m));
    }
    static EWF_DEV float pow(float x, float y) { return powf(x, y); }
    static EWF_DEV float pow_pos(float x, float y) { return powf(x, y); }
    static EWF_DEV float div(float x, float y) { return x / y; }
    static EWF_DEV float recip(float x) { return 1.0f / x; }
};

// native-rate flavour: hardware exp2 / log2 / rcp / sqrt with minimal fix-ups.  Relative
// error is a few float32 units for moderate arguments; meant for float16-stored results.
struct ewf_fast {
    static EWF_DEV float exp(float x) { return __builtin_amdgcn_exp2f(x * 1.44269504088896340736f); }
    static EWF_DEV float log(float x) { return __builtin_amdgcn_logf(x) * 0.69314718055994530942f; }
    static EWF_DEV float recip(float x) { return __builtin_amdgcn_rcpf(x); }
    static EWF_DEV float log1p(float x)
    {
        // log(u) * x / (u - 1) with u = fl(1 + x) cancels the rounding of 1 + x
        float u = 1.0f + x;
        float d = u - 1.0f;
        float l = log(u);
        return (d == 0.0f) ? x : l * (x * recip(d));
    }
    static EWF_DEV float expm1(float x)
    {
        float e = exp(x);
        return (fabsf(x) < 0.25f) ? x * (1.0f + x * (0.5f + x * (0.16666667f + x * (0.041666668f + x * 0.0083333338f))))
                                   : e - 1.0f;
    }
    static EWF_DEV float sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
    static EWF_DEV float sigmoid(float x) { return recip(1.0f + exp(-x)); }
    static EWF_DEV float tanh(float x)
    {
        float a = fabsf(x);
        a = (a > 15.0f) ? 15.0f : a;                  // a NaN stays (a min() would drop it)
        float e = exp(-2.0f * a);
        float t = (1.0f - e) * recip(1.0f + e);
        t = (a < 0.03125f) ? a * (1.0f - a * a * 0.33333334f) : t;
        return copysignf(t, x);
    }
    // base known to be positive (the generator proves it from the graph, e.g. x*x + 1)
    static EWF_DEV float pow_pos(float x, float y) { return __builtin_amdgcn_exp2f(y * __builtin_amdgcn_logf(x)); }
    // any base: |x|^y, then the sign rules for negative bases (integer exponents only) and
    // the convention pow(x, 0) = 1
    static EWF_DEV float pow(float x, float y)
    {
        float r = __builtin_amdgcn_exp2f(y * __builtin_amdgcn_logf(fabsf(x)));
        float t = truncf(y);
        float h = t * 0.5f;
        bool isint = (t == y);
        bool odd = isint && (truncf(h) != h);
        float neg = isint ? (odd ? -r : r) : __uint_as_float(0x7fc00000u);
        r = (x < 0.0f) ? neg : r;
        return (y == 0.0f) ? 1.0f : r;
    }
    static EWF_DEV float div(float x, float y) { return x * recip(y); }
};

// native-rate flavour without the fix-ups: log1p(x) = log(1 + x), expm1(x) = exp(x) - 1.
// Their absolute error near zero is about one float32 unit of 1.0 (6e-8): invisible once the
// result is rounded to float16 under an absolute + relative bound, and a third of the
// instructions.  Chosen automatically only when every output is stored as float16.
struct ewf_bare : ewf_fast {
    static EWF_DEV float log1p(float x) { return log(1.0f + x); }
    static EWF_DEV float expm1(float x) { return exp(x) - 1.0f; }
    static EWF_DEV float tanh(float x)
    {
        float e = exp(-2.0f * fabsf(x));
        return copysignf((1.0f - e) * recip(1.0f + e), x);
    }
};

// Tile coordinates come out of integer divisions, which run on the vector unit; telling the
// compiler that the value is the same in every lane moves all address bases derived from it
// to scalar registers.
EWF_DEV int ewf_uniform(int v) { return __builtin_amdgcn_readfirstlane(v); }
EWF_DEV long long ewf_uniform(long long v)
{
    unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(unsigned long long)v);
    unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((unsigned long long)v >> 32));
    return (long long)(((unsigned long long)hi << 32) | lo);
}

// Address of element `off` of a uniform base with 32-bit byte-offset arithmetic (the caller
// guarantees that the byte offset fits): lets the load use a scalar base plus a 32-bit lane
// offset instead of a 64-bit add per access.
template <typename T>
EWF_DEV T *ewf_at(T *base, unsigned off)
{
    return (T *)((char *)base + off * (unsigned)sizeof(T));
}
template <typename T>
EWF_DEV const T *ewf_at(const T *base, unsigned off)
{
    return (const T *)((const char *)base + off * (unsigned)sizeof(T));
}
template <typename T>
EWF_DEV T *ewf_at(T *base, long long off) { return base + off; }
template <typename T>
EWF_DEV const T *ewf_at(const T *base, long long off) { return base + off; }

// Product of two non-negative factors that the generator knows to be below 2^24: the masks
// let the compiler pick the full-rate 24-bit multiply.
EWF_DEV unsigned ewf_mul24(int a, int b)
{
    return ((unsigned)a & 0xffffffu) * ((unsigned)b & 0xffffffu);
}
EWF_DEV unsigned ewf_mul24(int a, long long b) { return ewf_mul24(a, (int)b); }

// ------------------------------------------------------------------ reductions

// Moves every 32-bit word of v through a DPP lane pattern.
template <int CTRL, typename T>
EWF_DEV T ewf_dpp(const T &v)
{
    static_assert(sizeof(T) % 4 == 0, "accumulator must be made of 32-bit words");
    T r;
    const int *src = reinterpret_cast<const int *>(&v);
    int *dst = reinterpret_cast<int *>(&r);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) / 4); i++)
        dst[i] = __builtin_amdgcn_update_dpp(src[i], src[i], CTRL, 0xf, 0xf, false);
    return r;
}

template <typename T>
EWF_DEV T ewf_lane_xor(const T &v, int mask)
{
    T r;
    const int *src = reinterpret_cast<const int *>(&v);
    int *dst = reinterpret_cast<int *>(&r);
#pragma unroll
    for (int i = 0; i < (int)(sizeof(T) / 4); i++) dst[i] = __shfl_xor(src[i], mask, 64);
    return r;
}

// All 64 lanes end with the combination of all 64 inputs.  The butterfly combines the same
// pairs on both partners, so with a commutative `op` every lane holds identical bits.
template <typename T, typename F>
EWF_DEV T ewf_wave_reduce(T v, F op)
{
    v = op(v, ewf_dpp<0xB1>(v));    // quad_perm [1,0,3,2]   : lane ^ 1
    v = op(v, ewf_dpp<0x4E>(v));    // quad_perm [2,3,0,1]   : lane ^ 2
    v = op(v, ewf_dpp<0x141>(v));   // row_half_mirror       : quads 0<->1, 2<->3
    v = op(v, ewf_dpp<0x140>(v));   // row_mirror            : half rows
    v = op(v, ewf_lane_xor(v, 16)); // rows 0<->1, 2<->3
    v = op(v, ewf_lane_xor(v, 32)); // row pairs
    return v;
}

// Workgroup reduction: wave butterflies, then the per-wave results are combined in wave
// order by every thread from LDS.  `smem` must hold NWAVES elements of T and may be reused
// after the call returns.
template <int NWAVES, typename T, typename F>
EWF_DEV T ewf_block_reduce(T v, F op, T *smem, int tid)
{
    v = ewf_wave_reduce(v, op);
    if (NWAVES == 1) return v;
    if ((tid & 63) == 0) smem[tid >> 6] = v;
    __syncthreads();
    T r = smem[0];
#pragma unroll
    for (int w = 1; w < NWAVES; w++) r = op(r, smem[w]);
    __syncthreads();
    return r;
}

// The same for a buffer that is written once per kernel (no loop around the call): the barrier
// that protects the buffer from the next round of writes is not needed.
template <int NWAVES, typename T, typename F>
EWF_DEV T ewf_block_reduce_once(T v, F op, T *smem, int tid)
{
    v = ewf_wave_reduce(v, op);
    if (NWAVES == 1) return v;
    if ((tid & 63) == 0) smem[tid >> 6] = v;
    __syncthreads();
    T r = smem[0];
#pragma unroll
    for (int w = 1; w < NWAVES; w++) r = op(r, smem[w]);
    return r;
}

// A maximum taken the cheap way (the hardware maximum drops NaN) next to a check word that turns
// NaN as soon as an element is NaN or infinite: the sum of the elements times zero.  While the
// check word is a number the maximum is the one the NaN-aware rules would have given.
struct ewf_fmax { float m, c; };
struct ewf_fmax_combine {
    EWF_DEV ewf_fmax operator()(const ewf_fmax &x, const ewf_fmax &y) const
    {
        ewf_fmax r;
        r.m = __builtin_fmaxf(x.m, y.m);
        r.c = x.c + y.c;
        return r;
    }
};
struct ewf_imin { EWF_DEV int operator()(int a, int b) const { return a < b ? a : b; } };

#endif  // EWF_PRELUDE_H
