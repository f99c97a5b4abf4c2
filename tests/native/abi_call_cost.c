/* A plain C caller of the library: times what one call of the C ABI costs on
 * the host (argument checks, order applied to the tables, one kernel launch)
 * without any binding around it, on the smallest configuration (K = 4 updates
 * of 1,048,576 binary32 elements, no momentum), where that cost is what a
 * caller sees.  Prints one line of JSON. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>

#include <stdio.h>
#include <stdlib.h>
#include <time.h>

#include "mlfabric.h"

#define CHECK(call)                                                        \
    do {                                                                   \
        hipError_t e_ = (call);                                            \
        if (e_ != hipSuccess) {                                            \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));     \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static double now_us(void)
{
    struct timespec ts;
    clock_gettime(CLOCK_MONOTONIC, &ts);
    return ts.tv_sec * 1e6 + ts.tv_nsec * 1e-3;
}

int main(void)
{
    enum { K = 4, CALLS = 2000 };
    const int64_t n = 1048576;
    const void *updates[K];
    float *model = NULL;
    const int32_t order[K] = {2, 0, 3, 1};
    const float weights[K] = {0.25f, 0.25f, 0.25f, 0.25f};
    hipStream_t stream;
    CHECK(hipSetDevice(0));
    CHECK(hipStreamCreate(&stream));
    for (int k = 0; k < K; ++k) {
        void *p = NULL;
        CHECK(hipMalloc(&p, (size_t)n * sizeof(float)));
        CHECK(hipMemsetAsync(p, 0, (size_t)n * sizeof(float), stream));
        updates[k] = p;
    }
    CHECK(hipMalloc((void **)&model, (size_t)n * sizeof(float)));
    CHECK(hipMemsetAsync(model, 0, (size_t)n * sizeof(float), stream));
    for (int i = 0; i < 20; ++i) {
        mlf_status st = mlf_aggregate_apply(model, NULL, NULL, updates, K, n, MLF_F32, order, K, weights,
                                            0.01f, 0.0f, stream);
        if (st != MLF_OK) {
            fprintf(stderr, "%s\n", mlf_status_string(st));
            return 1;
        }
    }
    CHECK(hipStreamSynchronize(stream));
    const double t0 = now_us();
    for (int i = 0; i < CALLS; ++i) {
        mlf_aggregate_apply(model, NULL, NULL, updates, K, n, MLF_F32, order, K, weights, 0.01f, 0.0f,
                            stream);
    }
    const double t1 = now_us();
    CHECK(hipStreamSynchronize(stream));
    const double t2 = now_us();
    /* the argument checks alone: n = 0 returns before anything is enqueued */
    const double t3 = now_us();
    for (int i = 0; i < CALLS; ++i) {
        mlf_aggregate_apply(model, NULL, NULL, updates, K, 0, MLF_F32, order, K, weights, 0.01f, 0.0f,
                            stream);
    }
    const double t4 = now_us();
    printf("{\"calls\": %d, \"host_us_per_call\": %.3f, \"us_per_call_until_done\": %.3f, "
           "\"checks_only_us_per_call\": %.3f}\n",
           CALLS, (t1 - t0) / CALLS, (t2 - t0) / CALLS, (t4 - t3) / CALLS);
    for (int k = 0; k < K; ++k) CHECK(hipFree((void *)updates[k]));
    CHECK(hipFree(model));
    CHECK(hipStreamDestroy(stream));
    return 0;
}
