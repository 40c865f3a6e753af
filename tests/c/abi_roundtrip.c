/*
 * A C11 program that uses the library the way a C caller would - no Python, no torch: device memory from the HIP
 * runtime, the optimiser through include/comp_ams.h.  It reads a problem from a binary file, runs the steps,
 * and writes the resulting state to another file; tests/test_gpu_c_caller.py feeds it seeded inputs and compares
 * what it wrote with the CPU oracle.
 *
 * input file:  int64 d, int64 n, int64 compressor, int64 k_or_block, int64 method, int64 steps,
 *              float theta0[d], then per step float grads[n][d]
 * output file: float theta[d], m[d], v[d], vhat[d], then (error feedback) e[n][d] or (CD-Adam) ghat[n][d]
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "comp_ams.h"

#define CHECK(call)                                                                       \
    do {                                                                                  \
        int rc__ = (call);                                                                \
        if (rc__ != COMP_AMS_OK) {                                                        \
            fprintf(stderr, "%s -> %d: %s\n", #call, rc__, comp_ams_last_error(h));       \
            return 2;                                                                     \
        }                                                                                 \
    } while (0)

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s problem.bin result.bin\n", argv[0]);
        return 1;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) return 1;
    int64_t hdr[6];
    if (fread(hdr, sizeof hdr[0], 6, in) != 6) return 1;
    const int64_t d = hdr[0], n = hdr[1], steps = hdr[5];
    const size_t row = (size_t)d, all = (size_t)n * row;
    float *host = (float *)malloc(all * sizeof(float));
    float *out = (float *)malloc(row * sizeof(float));
    if (!host || !out) return 1;

    comp_ams_t *h = NULL;
    CHECK(comp_ams_create(&h, d, (int32_t)n, (int32_t)hdr[2], hdr[3], 0.9f, 0.999f, 1e-8f, 1e-3f));
    CHECK(comp_ams_set_method(h, (int32_t)hdr[4]));
    if (fread(host, sizeof(float), row, in) != row) return 1;
    CHECK(comp_ams_set_theta(h, host, 0));

    float *grads_dev = NULL;
    hipStream_t stream = NULL;
    if (hipMalloc((void **)&grads_dev, all * sizeof(float)) != hipSuccess) return 3;
    if (hipStreamCreate(&stream) != hipSuccess) return 3;
    for (int64_t t = 0; t < steps; ++t) {
        if (fread(host, sizeof(float), all, in) != all) return 1;
        /* the copy is enqueued on the stream the step runs on; the host buffer is reused only after it is done */
        if (hipMemcpyAsync(grads_dev, host, all * sizeof(float), hipMemcpyHostToDevice, stream) != hipSuccess) return 3;
        if (hipStreamSynchronize(stream) != hipSuccess) return 3;
        CHECK(comp_ams_step(h, grads_dev, stream));
    }
    fclose(in);

    FILE *res = fopen(argv[2], "wb");
    if (!res) return 1;
    CHECK(comp_ams_get_theta(h, out, 0));
    fwrite(out, sizeof(float), row, res);
    CHECK(comp_ams_get_m(h, out, 0));
    fwrite(out, sizeof(float), row, res);
    CHECK(comp_ams_get_v(h, out, 0));
    fwrite(out, sizeof(float), row, res);
    CHECK(comp_ams_get_vhat(h, out, 0));
    fwrite(out, sizeof(float), row, res);
    for (int32_t i = 0; i < (int32_t)n; ++i) {
        if (hdr[4] == COMP_AMS_METHOD_EF)
            CHECK(comp_ams_get_error(h, i, out, 0));
        else if (hdr[4] == COMP_AMS_METHOD_CD)
            CHECK(comp_ams_get_ghat_worker(h, i, out, 0));
        else
            break;
        fwrite(out, sizeof(float), row, res);
    }
    fclose(res);
    comp_ams_destroy(h);
    (void)hipStreamDestroy(stream);
    (void)hipFree(grads_dev);
    free(host);
    free(out);
    printf("abi roundtrip: %lld steps done\n", (long long)steps);
    return 0;
}
