/*
 * A C99 client of libwagma: no Python, no C++.  Reads a problem from a file, runs
 * wagma_create -> wagma_step x iters -> wagma_destroy on the GPU through include/wagma.h and the
 * HIP runtime's C API, and writes w, m and pub back.  tests/test_gpu_c_client.py compares the
 * bytes with the CPU oracle.
 *
 * Input file (little endian):  int32 P, S, tau, iters;  int64 n;  float lr, mu;
 *   then w, m, pub: P x n floats each (rows without padding);
 *   then per iteration: ceil(P/64) uint64 mask words, followed by g: P x n floats.
 * Output file: w, m, pub: P x n floats each.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "wagma.h"

#define CHECK_HIP(call)                                                              \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s failed: %s\n", #call, hipGetErrorString(e_));        \
            return 2;                                                                \
        }                                                                            \
    } while (0)

#define CHECK_WAGMA(call)                                                            \
    do {                                                                             \
        int rc_ = (call);                                                            \
        if (rc_ != WAGMA_OK) {                                                       \
            fprintf(stderr, "%s failed: %s\n", #call, wagma_strerror(rc_));          \
            return 3;                                                                \
        }                                                                            \
    } while (0)

/* rows of n floats in the file <-> rows of ld floats on the device */
static int upload(float *dev, const float *host, int P, int64_t n, int64_t ld)
{
    CHECK_HIP(hipMemcpy2D(dev, (size_t)ld * sizeof(float), host, (size_t)n * sizeof(float),
                          (size_t)n * sizeof(float), (size_t)P, hipMemcpyHostToDevice));
    return 0;
}

static int download(float *host, const float *dev, int P, int64_t n, int64_t ld)
{
    CHECK_HIP(hipMemcpy2D(host, (size_t)n * sizeof(float), dev, (size_t)ld * sizeof(float),
                          (size_t)n * sizeof(float), (size_t)P, hipMemcpyDeviceToHost));
    return 0;
}

int main(int argc, char **argv)
{
    if (argc != 3) {
        fprintf(stderr, "usage: %s problem.bin result.bin\n", argv[0]);
        return 1;
    }
    FILE *in = fopen(argv[1], "rb");
    if (!in) {
        perror(argv[1]);
        return 1;
    }
    int32_t head[4];
    int64_t n;
    float rates[2];
    if (fread(head, sizeof(int32_t), 4, in) != 4 || fread(&n, sizeof n, 1, in) != 1 ||
        fread(rates, sizeof(float), 2, in) != 2) {
        fprintf(stderr, "short header\n");
        return 1;
    }
    const int P = head[0], S = head[1], tau = head[2], iters = head[3];
    const int words = (P + 63) / 64;
    const size_t count = (size_t)P * (size_t)n;
    float *host = (float *)malloc(count * sizeof(float));
    uint64_t mask[WAGMA_MAX_P / 64];
    if (!host)
        return 1;

    wagma_ctx *ctx = NULL;
    CHECK_WAGMA(wagma_create(&ctx, P, S, n, tau));
    const int64_t ld = wagma_row_stride(ctx);
    float *w, *g, *m, *pub;
    const size_t bytes = (size_t)P * (size_t)ld * sizeof(float);
    CHECK_HIP(hipMalloc((void **)&w, bytes));
    CHECK_HIP(hipMalloc((void **)&g, bytes));
    CHECK_HIP(hipMalloc((void **)&m, bytes));
    CHECK_HIP(hipMalloc((void **)&pub, bytes));
    CHECK_HIP(hipMemset(g, 0, bytes));
    float *state[3];
    state[0] = w;
    state[1] = m;
    state[2] = pub;
    for (int k = 0; k < 3; ++k) {
        CHECK_HIP(hipMemset(state[k], 0, bytes));
        if (fread(host, sizeof(float), count, in) != count)
            return 1;
        if (upload(state[k], host, P, n, ld))
            return 2;
    }

    const int32_t *schedule = NULL;
    for (int t = 0; t < iters; ++t) {
        if (fread(mask, sizeof(uint64_t), (size_t)words, in) != (size_t)words ||
            fread(host, sizeof(float), count, in) != count)
            return 1;
        if (upload(g, host, P, n, ld))
            return 2;
        CHECK_WAGMA(wagma_group_schedule(ctx, t, NULL, &schedule));
        printf("t=%d %s first group:", t, wagma_is_global_iteration(ctx, t) ? "global" : "group ");
        for (int e = 0; e < S && e < 8; ++e)
            printf(" %d", (int)schedule[e]);
        printf("\n");
        CHECK_WAGMA(wagma_step(ctx, w, g, m, pub, mask, rates[0], rates[1], t, NULL));
        CHECK_HIP(hipDeviceSynchronize());
    }
    fclose(in);

    FILE *out = fopen(argv[2], "wb");
    if (!out) {
        perror(argv[2]);
        return 1;
    }
    for (int k = 0; k < 3; ++k) {
        if (download(host, state[k], P, n, ld))
            return 2;
        if (fwrite(host, sizeof(float), count, out) != count)
            return 1;
    }
    fclose(out);
    CHECK_WAGMA(wagma_destroy(ctx));
    CHECK_HIP(hipFree(w));
    CHECK_HIP(hipFree(g));
    CHECK_HIP(hipFree(m));
    CHECK_HIP(hipFree(pub));
    free(host);
    printf("c client: done\n");
    return 0;
}
