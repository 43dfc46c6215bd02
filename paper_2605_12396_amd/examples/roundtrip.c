/*
 * roundtrip.c -- the library called from plain C through its C ABI (no Python, no torch): compress an fp32 message
 * on the GPU, decompress it, check the error bound, then reduce the stream with itself and check that the result
 * decodes to twice the values.  Build (from the repository root):
 *
 *   gcc -std=c99 -D__HIP_PLATFORM_AMD__ -I/opt/rocm/include -Iinclude paper_2605_12396_amd/examples/roundtrip.c \
 *       -Lpaper_2605_12396_amd -lnz -L/opt/rocm/lib -lamdhip64 -lm -Wl,-rpath,$PWD/paper_2605_12396_amd -o roundtrip
 *
 * Exit status 0 = all checks passed.
 */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "nz.h"

#define CHECK_HIP(e) do { hipError_t err_ = (e); if (err_ != hipSuccess) { fprintf(stderr, "HIP error %d at line %d\n", (int)err_, __LINE__); return 10; } } while (0)

int main(void) {
    const size_t n = 1000003;                       /* a ragged last frame */
    const float eb = 1e-4f;
    nz_opts opts;
    memset(&opts, 0, sizeof opts);                  /* defaults: 262144-element frames, alphabet 256 */
    opts.force_codec = -1;

    float* x = (float*)malloc(4 * n); float* y = (float*)malloc(4 * n);
    if (!x || !y) return 1;
    unsigned s = 12345u;                            /* a peaked synthetic message: sums of small uniform draws */
    for (size_t i = 0; i < n; i++) {
        float a = 0.0f;
        for (int k = 0; k < 4; k++) { s = s * 1664525u + 1013904223u; a += (float)(s >> 8) / 16777216.0f - 0.5f; }
        x[i] = 2e-3f * a;
    }

    const size_t cap = nz_compress_bound(n, &opts), wsb = nz_reduce_workspace_bytes(n, &opts);
    if (!cap || !wsb) return 2;
    float *d_x, *d_y; void *d_stream, *d_sum, *d_ws; nz_result* d_res; nz_result res;
    CHECK_HIP(hipMalloc((void**)&d_x, 4 * n)); CHECK_HIP(hipMalloc((void**)&d_y, 4 * n));
    CHECK_HIP(hipMalloc(&d_stream, cap)); CHECK_HIP(hipMalloc(&d_sum, cap)); CHECK_HIP(hipMalloc(&d_ws, wsb));
    CHECK_HIP(hipMalloc((void**)&d_res, sizeof(nz_result)));
    CHECK_HIP(hipMemcpy(d_x, x, 4 * n, hipMemcpyHostToDevice));

    if (nz_compress(d_x, n, eb, d_stream, cap, d_res, &opts, d_ws, wsb, NULL) != NZ_OK) return 3;
    CHECK_HIP(hipMemcpy(&res, d_res, sizeof res, hipMemcpyDeviceToHost));      /* (synchronises with the null stream) */
    if (res.status != NZ_OK || res.bytes == 0) return 4;
    const size_t bytes = (size_t)res.bytes;
    printf("compressed %zu fp32 values to %zu bytes (ratio %.2f; frames raw/fixed/huffman %u/%u/%u)\n", n, bytes,
           4.0 * (double)n / (double)bytes, res.n_raw, res.n_fixed, res.n_huff);

    if (nz_decompress(d_stream, bytes, d_y, n, eb, d_res, &opts, d_ws, wsb, NULL) != NZ_OK) return 5;
    CHECK_HIP(hipMemcpy(&res, d_res, sizeof res, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(y, d_y, 4 * n, hipMemcpyDeviceToHost));
    if (res.status != NZ_OK) return 6;
    double worst = 0.0;
    for (size_t i = 0; i < n; i++) { double e = fabs((double)x[i] - (double)y[i]); if (e > worst) worst = e; }
    printf("largest error %.3g (bound %.3g)\n", worst, (double)eb);
    if (worst > (double)eb) return 7;

    /* the stream reduced with itself decodes to exactly twice the decompressed values (integer codes add exactly) */
    if (nz_reduce_frames(d_stream, bytes, d_stream, bytes, d_sum, cap, n, eb, d_res, &opts, d_ws, wsb, NULL) != NZ_OK) return 8;
    CHECK_HIP(hipMemcpy(&res, d_res, sizeof res, hipMemcpyDeviceToHost));
    if (res.status != NZ_OK) return 9;
    const size_t sum_bytes = (size_t)res.bytes;
    if (nz_decompress(d_sum, sum_bytes, d_x, n, eb, d_res, &opts, d_ws, wsb, NULL) != NZ_OK) return 11;
    CHECK_HIP(hipMemcpy(x, d_x, 4 * n, hipMemcpyDeviceToHost));
    for (size_t i = 0; i < n; i++) if (x[i] != 2.0f * y[i]) { fprintf(stderr, "element %zu: %g != 2 * %g\n", i, x[i], y[i]); return 12; }
    printf("reduced stream: %zu bytes, decodes to twice the values\n", sum_bytes);

    hipFree(d_x); hipFree(d_y); hipFree(d_stream); hipFree(d_sum); hipFree(d_ws); hipFree(d_res);
    free(x); free(y);
    return 0;
}
