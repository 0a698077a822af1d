// Small ahead-of-time device code for gfx950: a zero fill for workspace bookkeeping (a fill
// kernel rather than a memset so that callers may record it into a HIP graph), the plain
// dwordx4 grid-stride copy that bandwidth figures are quoted against, and the library's own
// static workspace with the entry point that uses it.
#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>
#include <mutex>

#include "ewf_internal.h"

namespace ewf {

__global__ void __launch_bounds__(256) k_fill_zero(uint4 *p, size_t n16, unsigned char *tail, size_t ntail)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
    if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

// The plain copy, as a measured ceiling for streaming kernels: a workgroup owns one contiguous,
// line-aligned piece of UNROLL * 4 KiB and makes a single trip over it: every thread issues its
// UNROLL 16-byte loads (each instruction covers 4 KiB contiguous across the workgroup), then its
// stores; the data is touched once, so both are non-temporal.  Workgroup w takes piece w, so
// neighbouring pieces are in flight at the same time.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <int UNROLL>
__global__ void __launch_bounds__(256) k_copy(u32x4 *__restrict__ dst, const u32x4 *__restrict__ src, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * (256 * UNROLL) + threadIdx.x;
    u32x4 v[UNROLL];
    if (base - threadIdx.x + 256 * UNROLL <= n16) {          // a whole piece: no test between the loads
#pragma unroll
        for (int u = 0; u < UNROLL; u++) v[u] = __builtin_nontemporal_load(src + base + (size_t)u * 256);
#pragma unroll
        for (int u = 0; u < UNROLL; u++) __builtin_nontemporal_store(v[u], dst + base + (size_t)u * 256);
    } else {
#pragma unroll
        for (int u = 0; u < UNROLL; u++) {
            const size_t i = base + (size_t)u * 256;
            if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
        }
    }
}

// Fills a strided n-d view with one 2- or 4-byte pattern (the identity of a reduction over an
// empty axis).
struct FillView { long long shape[8]; long long strides[8]; int rank; };

template <typename T>
__global__ void __launch_bounds__(256) k_fill_view(T *p, FillView v, long long total, T value)
{
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
        long long r = i, off = 0;
        for (int d = v.rank - 1; d >= 0; d--) { off += (r % v.shape[d]) * v.strides[d]; r /= v.shape[d]; }
        p[off] = value;
    }
}

void aux_fill_view(void *ptr, int rank, const int64_t *shape, const int64_t *strides, int elem_bytes, uint32_t bits,
                   hipStream_t stream)
{
    FillView v;
    long long total = 1;
    v.rank = rank;
    for (int d = 0; d < rank; d++) { v.shape[d] = shape[d]; v.strides[d] = strides[d]; total *= shape[d]; }
    if (total <= 0) return;
    unsigned blocks = (unsigned)((total + 255) / 256);
    if (blocks > 4096) blocks = 4096;
    if (elem_bytes == 2)
        hipLaunchKernelGGL(k_fill_view<unsigned short>, dim3(blocks), dim3(256), 0, stream, (unsigned short *)ptr, v, total, (unsigned short)bits);
    else
        hipLaunchKernelGGL(k_fill_view<unsigned int>, dim3(blocks), dim3(256), 0, stream, (unsigned int *)ptr, v, total, bits);
}

void aux_fill_zero(void *ptr, size_t nbytes, hipStream_t stream)
{
    size_t n16 = nbytes / 16, ntail = nbytes % 16;
    unsigned blocks = (unsigned)((n16 + 255) / 256);
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, stream, (uint4 *)ptr, n16,
                       (unsigned char *)ptr + n16 * 16, ntail);
}

void aux_copy(void *dst, const void *src, size_t nbytes, hipStream_t stream)
{
    // one 16-byte access per thread, 4 KiB per workgroup: the fastest of 1, 2, 4 and 8 accesses per
    // thread on 411 MB (123.6, 130.2, 133.6 and 127.5 us; with ordinary instead of non-temporal
    // accesses 134.9 us and more; the runtime's own device-to-device copy 155 us)
    constexpr int kUnroll = 1;
    const size_t n16 = nbytes / 16;
    const size_t per_block = (size_t)256 * kUnroll;
    const size_t blocks = (n16 + per_block - 1) / per_block;
    if (blocks == 0 || blocks > 0x7fffffffu) return;         // (beyond 16 TiB: not a size this call is used for)
    hipLaunchKernelGGL(k_copy<kUnroll>, dim3((unsigned)blocks), dim3(256), 0, stream, (u32x4 *)dst, (const u32x4 *)src, n16);
}

}  // namespace ewf

// =========================================================================================
// ewf_run_static: ewf_run for callers that cannot allocate device memory.
//
// The workspace (partial results of reductions split over workgroups, temporaries of plans in
// several passes) lives in `scratch`, a static device array that every GPU the library runs on
// holds until the process ends.  In host code the array's name is only a handle for the symbol,
// not a device address: its address on the current device is asked for once per device and kept;
// everything that touches the memory -- kernel arguments here -- uses that address.

static __device__ __align__(256) unsigned char scratch[EWF_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {nullptr};

// Address of `scratch` on the current device (looked up on the first call per device).
ewf_status static_workspace(void **ptr)
{
    int dev = -1;
    hipError_t he = hipGetDevice(&dev);
    if (he != hipSuccess) { ewf::set_error("no HIP device: %s", hipGetErrorString(he)); return EWF_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) { ewf::set_error("device ordinal %d is beyond the %d this entry point supports", dev, kMaxDevices); return EWF_EINVAL; }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        he = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (he != hipSuccess || !p) {
            ewf::set_error("hipGetSymbolAddress(static workspace): %s", hipGetErrorString(he));
            return EWF_EHIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return EWF_OK;
}

}  // namespace

extern "C" ewf_status ewf_run_static(ewf_exec *e, const ewf_tensor *in, int32_t nin, const double *scalars, int32_t nscalars,
                                     const ewf_tensor *out, int32_t nout, void *hip_stream)
{
    return ewf::guarded([&]() -> ewf_status {
        if (!e) { ewf::set_error("null executable"); return EWF_EINVAL; }
        // the layout must have been planned (ewf_plan compiles and, with a device current, loads the
        // kernels): nothing is compiled, loaded or allocated from here on
        ewf::Plan *p = nullptr;
        ewf_status st = ewf::make_plan(e->e, in, nin, out, nout, &p, /*lookup_only=*/true);
        if (st != EWF_OK) return st;
        if (p->workspace_bytes > (size_t)EWF_STATIC_WORKSPACE_BYTES) {
            ewf::set_error("this layout needs a workspace of %zu bytes, the static one holds %zu: use ewf_run with a workspace of your own",
                           p->workspace_bytes, (size_t)EWF_STATIC_WORKSPACE_BYTES);
            return EWF_ENOMEM;
        }
        void *ws = nullptr;
        st = static_workspace(&ws);
        if (st != EWF_OK) return st;
        // (the kernels write every workspace word before they read it: what the previous call left
        // in the array needs no clearing)
        return ewf::run_exec(e->e, in, nin, scalars, nscalars, out, nout, ws, (size_t)EWF_STATIC_WORKSPACE_BYTES, hip_stream,
                             /*no_setup=*/true);
    });
}
