/* Test driver for the host side of the C ABI: argument checks and scratch-size
 * queries, which return before anything is enqueued, so it runs without a GPU.
 * tests/test_abi_sanitizers.py builds the library's host code with
 * AddressSanitizer and UndefinedBehaviorSanitizer and links this file to it. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "mlfabric.h"

#define EXPECT(call, want)                                                              \
    do {                                                                                \
        int got_ = (int)(call);                                                         \
        if (got_ != (int)(want)) {                                                      \
            printf("line %d: %s = %d, want %d\n", __LINE__, #call, got_, (int)(want)); \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

int main(void)
{
    /* addresses that are never dereferenced by the checks */
    float *fake = (float *)(uintptr_t)0x7f0000000000ull;
    const void *ups[MLF_MAX_K + 1];
    for (int k = 0; k <= MLF_MAX_K; ++k) ups[k] = (const char *)fake + ((size_t)(k + 4) << 24);
    int32_t order[MLF_MAX_K + 1];
    for (int k = 0; k <= MLF_MAX_K; ++k) order[k] = k;
    float weights[MLF_MAX_K + 1] = {0};
    int32_t lens[4] = {1, 1, 2, 0};
    int32_t twice[2] = {1, 1}, outside[2] = {0, 9};

    EXPECT(mlf_aggregate(NULL, 2, 8, MLF_F32, order, 2, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 0, 8, MLF_F32, order, 0, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, MLF_MAX_K + 1, 8, MLF_F32, order, 2, NULL, fake, NULL), MLF_EUNSUPPORTED);
    EXPECT(mlf_aggregate(ups, 2, -1, MLF_F32, order, 2, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 2, 8, MLF_F32, twice, 2, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 2, 8, MLF_F32, outside, 2, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 2, 8, MLF_F32, order, 3, NULL, fake, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 2, 8, MLF_F32, order, 2, weights, NULL, NULL), MLF_EINVAL);
    EXPECT(mlf_aggregate(ups, 2, 0, MLF_F32, order, 2, weights, fake, NULL), MLF_OK);
    EXPECT(mlf_apply_ordered(NULL, NULL, ups, 2, 8, MLF_F32, order, 2, 0.1f, 0.9f, NULL), MLF_EINVAL);
    EXPECT(mlf_apply_ordered(fake, NULL, ups, 2, 8, MLF_BF16, order, 0, 0.1f, 0.9f, NULL), MLF_OK);
    EXPECT(mlf_aggregate_apply(NULL, NULL, NULL, ups, 2, 8, MLF_F32, order, 2, NULL, 0.1f, 0.9f, NULL),
           MLF_EINVAL);
    EXPECT(mlf_apply_grouped(fake, NULL, ups, 4, 8, MLF_F32, order, 4, NULL, lens, 4, 0.1f, 0.9f, NULL),
           MLF_EINVAL);                                    /* a length of 0 */
    EXPECT(mlf_apply_grouped(fake, NULL, ups, 4, 8, MLF_F32, order, 4, NULL, lens, 2, 0.1f, 0.9f, NULL),
           MLF_EINVAL);                                    /* lengths add up to 2, not 4 */
    EXPECT(mlf_apply_grouped(fake, NULL, ups, 4, 0, MLF_F32, order, 4, NULL, lens, 3, 0.1f, 0.9f, NULL),
           MLF_OK);
    EXPECT(mlf_divergence(fake, fake, 8, NULL, NULL, 0, NULL), MLF_EINVAL);

    const int32_t *bufs[MLF_MAX_K + 1];
    int64_t counts_per[MLF_MAX_K + 1];
    for (int k = 0; k <= MLF_MAX_K; ++k) {
        bufs[k] = (const int32_t *)ups[k];
        counts_per[k] = 1;
    }
    int64_t negative[1] = {-1}, none[1] = {0};
    EXPECT(mlf_sparse_scatter_add(NULL, NULL, 3, 2, bufs, counts_per, 1, NULL, 0, NULL, NULL), MLF_EINVAL);
    EXPECT(mlf_sparse_scatter_add((int32_t *)fake, NULL, 3, 2, bufs, negative, 1, NULL, 0, NULL, NULL),
           MLF_EINVAL);
    EXPECT(mlf_sparse_scatter_add((int32_t *)fake, NULL, 3, 2, bufs, counts_per, MLF_MAX_K + 1, NULL, 0,
                                  NULL, NULL),
           MLF_EUNSUPPORTED);
    EXPECT(mlf_sparse_scatter_add((int32_t *)fake, NULL, 3, 2, bufs, none, 1, NULL, 0, NULL, NULL), MLF_OK);
    EXPECT(mlf_counts_add_dense((int32_t *)fake, NULL, 3, 2, bufs, 0, NULL), MLF_OK);
    EXPECT(mlf_counts_add_dense(NULL, NULL, 3, 2, bufs, 1, NULL), MLF_EINVAL);

    /* scratch sizes: extreme arguments must not overflow anything */
    const int32_t big = 2147483647;
    volatile size_t sink = 0;
    sink += mlf_sparse_workspace_bytes(big, big, INT64_MAX);
    sink += mlf_sparse_workspace_bytes(big, 1, INT64_MAX);
    sink += mlf_sparse_workspace_bytes(32768, 32768, 2147483647ll);
    sink += mlf_sparse_workspace_bytes(100000, 1000, 64000000);
    sink += mlf_sparse_workspace_bytes(-1, -1, -1);
    sink += mlf_norms_workspace_bytes(INT64_MAX);
    sink += mlf_norms_workspace_bytes(-1);
    sink += mlf_norms_workspace_bytes(61100840);
    for (int st = -99; st <= 5; ++st) {
        if (mlf_status_string((mlf_status)st) == NULL) return 1;
    }
    puts("abi sanitizer run: ok");
    return 0;
}
