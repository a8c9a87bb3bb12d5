/*
 * libhfr from plain C: the intra-node reduce of Algorithm 1 (K per-GPU copies of
 * a gradient chunk summed in GPU-index order) followed by the inter-node step of
 * Algorithm 2, pass 1 (add the neighbour's partial, then average), on buffers the
 * program allocates itself with the HIP runtime: the K copies and the node's
 * partial are carved from one allocation at the distance hfr_peer_stride gives,
 * as a staging arena would be. No Python, no torch.
 *
 * The inputs are small integers stored as fp32, so every partial sum is exact
 * and the expected result can be written down without any rounding question.
 *
 * Build (done by paper_2408_14158_amd/build.py):
 *   gcc -std=c99 c_abi_example.c -I<repo>/include -I/opt/rocm/include -D__HIP_PLATFORM_AMD__
 *       -L<dir of libhfr.so> -lhfr -L/opt/rocm/lib -lamdhip64 -Wl,-rpath,...
 * Run on a machine with an MI355X; exit status 0 and "ok" on success.
 */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>

#include "hfr.h"

#define K 8
#define CHECK_HIP(x)                                                                 \
    do {                                                                             \
        hipError_t e_ = (x);                                                         \
        if (e_ != hipSuccess) {                                                      \
            fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));                  \
            return 2;                                                                \
        }                                                                            \
    } while (0)
#define CHECK_HFR(x)                                                                 \
    do {                                                                             \
        hfr_status s_ = (x);                                                         \
        if (s_ != HFR_OK) {                                                          \
            fprintf(stderr, "%s: %s %s\n", #x, hfr_status_string(s_), hfr_last_error()); \
            return 3;                                                                \
        }                                                                            \
    } while (0)

int main(void) {
    const size_t n = ((size_t)6 << 20) + 13; /* 24 MiB per buffer: bulk launch shape, ragged end */
    const float scale = 1.0f / 16.0f;        /* exact */
    float* host = (float*)malloc(n * sizeof(float));
    const void* in[K];
    void *remote = NULL, *partial = NULL, *result = NULL, *arena = NULL;
    size_t stride;
    hipStream_t stream;
    int cus = 0, khz = 0, bits = 0, j;
    size_t i, bad = 0;

    if (!host) return 1;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_HFR(hfr_device_info(&cus, &khz, &bits));
    printf("libhfr %d on a device with %d compute units\n", hfr_version(), cus);

    stride = hfr_peer_stride(n * sizeof(float));
    if (stride < n * sizeof(float)) return 1;
    CHECK_HIP(hipMalloc(&arena, stride * (K + 1)));
    printf("K + 1 buffers of %zu bytes at a distance of %zu bytes\n", n * sizeof(float), stride);
    for (j = 0; j < K; ++j) {
        void* d = (char*)arena + (size_t)j * stride;
        for (i = 0; i < n; ++i) host[i] = (float)((i + 3u * (unsigned)j) % 7u) - 3.0f; /* -3 .. 3 */
        CHECK_HIP(hipMemcpy(d, host, n * sizeof(float), hipMemcpyHostToDevice));
        in[j] = d;
    }
    partial = (char*)arena + (size_t)K * stride;
    for (i = 0; i < n; ++i) host[i] = (float)(i % 5u); /* the neighbouring node's partial */
    CHECK_HIP(hipMalloc(&remote, n * sizeof(float)));
    CHECK_HIP(hipMemcpy(remote, host, n * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMalloc(&result, n * sizeof(float)));

    /* Algorithm 1, then Algorithm 2 pass 1 with the average */
    CHECK_HFR(hfr_reduce_sum(in, K, partial, n, HFR_F32, stream));
    CHECK_HFR(hfr_combine_avg(partial, remote, result, n, scale, HFR_F32, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(host, result, n * sizeof(float), hipMemcpyDeviceToHost));
    for (i = 0; i < n; ++i) {
        float want = 0.0f;
        for (j = 0; j < K; ++j) want += (float)((i + 3u * (unsigned)j) % 7u) - 3.0f;
        want = (want + (float)(i % 5u)) * scale;
        if (host[i] != want) ++bad;
    }
    /* the same in one pass over memory */
    CHECK_HFR(hfr_reduce_combine_avg(in, K, remote, partial, n, scale, HFR_F32, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    {
        float* again = (float*)malloc(n * sizeof(float));
        if (!again) return 1;
        CHECK_HIP(hipMemcpy(again, partial, n * sizeof(float), hipMemcpyDeviceToHost));
        for (i = 0; i < n; ++i)
            if (again[i] != host[i]) ++bad;
        free(again);
    }
    CHECK_HFR(hfr_shutdown());
    CHECK_HIP(hipFree(arena));
    CHECK_HIP(hipFree(remote));
    CHECK_HIP(hipFree(result));
    CHECK_HIP(hipStreamDestroy(stream));
    free(host);
    if (bad) {
        fprintf(stderr, "%zu mismatching elements\n", bad);
        return 4;
    }
    printf("ok: %zu elements, K=%d\n", n, K);
    return 0;
}
