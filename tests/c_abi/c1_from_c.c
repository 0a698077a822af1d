/*
 * The library used from plain C, without PyTorch: describes out = tanh(a * X + b) (X [rows, cols],
 * b [1, cols] broadcast over the rows, a a run-time scalar) and a per-column sum of the result
 * through the C ABI of include/ewf.h, runs it on buffers from hipMalloc, and writes inputs and
 * outputs as raw little-endian files that the test compares with the CPU oracle.
 *
 *   c1_from_c <rows> <cols> <a> <output directory>
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "ewf.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_EWF(x) do { ewf_status s_ = (x); if (s_ < 0) { fprintf(stderr, "%s: status %d: %s\n", #x, (int)s_, ewf_last_error()); return 3; } } while (0)

static int dump(const char *dir, const char *name, const void *data, size_t nbytes)
{
    char path[1024];
    snprintf(path, sizeof path, "%s/%s", dir, name);
    FILE *f = fopen(path, "wb");
    if (!f) return -1;
    size_t n = fwrite(data, 1, nbytes, f);
    fclose(f);
    return n == nbytes ? 0 : -1;
}

int main(int argc, char **argv)
{
    if (argc != 5) { fprintf(stderr, "usage: %s rows cols a outdir\n", argv[0]); return 1; }
    const int64_t rows = atoll(argv[1]), cols = atoll(argv[2]);
    const double a = atof(argv[3]);
    const char *dir = argv[4];

    /* describe: typed inputs, a run-time scalar, apply nodes, one reduction, two outputs */
    ewf_graph *g = NULL;
    CHECK_EWF(ewf_graph_create(2, &g));
    const uint8_t full[2] = {0, 0}, row_vector[2] = {1, 0};
    ewf_value x = ewf_input(g, EWF_F32, full);
    ewf_value b = ewf_input(g, EWF_F32, row_vector);
    ewf_value s = ewf_scalar(g, EWF_F32);
    ewf_value args[2];
    args[0] = s; args[1] = x;
    ewf_value ax = ewf_apply(g, EWF_MUL, args, 2);
    args[0] = ax; args[1] = b;
    ewf_value z = ewf_apply(g, EWF_ADD, args, 2);
    ewf_value y = ewf_apply(g, EWF_TANH, &z, 1);
    const int32_t axis0 = 0;
    ewf_value colsum = ewf_reduce(g, EWF_RSUM, y, &axis0, 1, 0);
    CHECK_EWF(x < 0 ? x : b < 0 ? b : s < 0 ? s : ax < 0 ? ax : z < 0 ? z : y < 0 ? y : colsum < 0 ? colsum : 0);
    CHECK_EWF(ewf_output(g, y, EWF_F32));
    CHECK_EWF(ewf_output(g, colsum, EWF_F32));
    ewf_exec *ex = NULL;
    CHECK_EWF(ewf_compile(g, NULL, &ex));
    ewf_graph_destroy(g);

    /* host data: a fixed linear congruential sequence in [-1, 1) */
    const size_t n = (size_t)(rows * cols);
    float *hx = (float *)malloc(n * 4), *hb = (float *)malloc((size_t)cols * 4);
    float *hy = (float *)malloc(n * 4), *hs = (float *)malloc((size_t)cols * 4);
    if (!hx || !hb || !hy || !hs) return 4;
    uint32_t state = 160502688u;
    for (size_t i = 0; i < n; i++) { state = state * 1664525u + 1013904223u; hx[i] = (float)(state >> 8) / 8388608.0f - 1.0f; }
    for (int64_t i = 0; i < cols; i++) { state = state * 1664525u + 1013904223u; hb[i] = (float)(state >> 8) / 8388608.0f - 1.0f; }

    float *dx, *db, *dy, *ds;
    CHECK_HIP(hipMalloc((void **)&dx, n * 4));
    CHECK_HIP(hipMalloc((void **)&db, (size_t)cols * 4));
    CHECK_HIP(hipMalloc((void **)&dy, n * 4));
    CHECK_HIP(hipMalloc((void **)&ds, (size_t)cols * 4));
    CHECK_HIP(hipMemcpy(dx, hx, n * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(db, hb, (size_t)cols * 4, hipMemcpyHostToDevice));

    const int64_t shape_x[2] = {rows, cols}, stride_x[2] = {cols, 1};
    const int64_t shape_b[2] = {1, cols}, stride_b[2] = {cols, 1};
    const int64_t shape_s[1] = {cols}, stride_s[1] = {1};
    ewf_tensor in[2] = {{dx, shape_x, stride_x}, {db, shape_b, stride_b}};
    ewf_tensor out[2] = {{dy, shape_x, stride_x}, {ds, shape_s, stride_s}};

    /* plan (compiles the kernel), allocate the workspace it asks for, run on a stream */
    int32_t rank = 0;
    int64_t oshape[EWF_MAX_DIMS];
    CHECK_EWF(ewf_output_shape(ex, in, 2, 1, &rank, oshape));
    if (rank != 1 || oshape[0] != cols) { fprintf(stderr, "unexpected shape of the column sums\n"); return 5; }
    size_t ws_bytes = 0;
    CHECK_EWF(ewf_plan(ex, in, 2, out, 2, &ws_bytes));
    void *ws = NULL;
    if (ws_bytes) CHECK_HIP(hipMalloc(&ws, ws_bytes));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    const double scalars[1] = {a};
    for (int rep = 0; rep < 3; rep++)                  /* the plan is reused: nothing is compiled again */
        CHECK_EWF(ewf_run(ex, in, 2, scalars, 1, out, 2, ws, ws_bytes, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    if (ewf_debug_compile_count(ex) != 1) { fprintf(stderr, "the kernel was compiled more than once\n"); return 6; }
    ewf_plan_info info;
    CHECK_EWF(ewf_debug_plan_info(ex, &info));

    CHECK_HIP(hipMemcpy(hy, dy, n * 4, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hs, ds, (size_t)cols * 4, hipMemcpyDeviceToHost));
    if (dump(dir, "x.bin", hx, n * 4) || dump(dir, "b.bin", hb, (size_t)cols * 4) || dump(dir, "y.bin", hy, n * 4) ||
        dump(dir, "colsum.bin", hs, (size_t)cols * 4)) { fprintf(stderr, "cannot write to %s\n", dir); return 7; }
    printf("kernel_class %d workspace %zu\n", (int)info.kernel_class, ws_bytes);

    ewf_exec_destroy(ex);
    CHECK_HIP(hipStreamDestroy(stream));
    hipFree(dx); hipFree(db); hipFree(dy); hipFree(ds); if (ws) hipFree(ws);
    free(hx); free(hb); free(hy); free(hs);
    return 0;
}
