/* Test driver: calls every entry point of the CPU oracle on exact-size heap
 * buffers.  Built with -fsanitize=address,undefined by
 * tests/test_oracle_sanitizers.py, so an out-of-bounds access, a signed
 * overflow or a misaligned access in the oracle ends the run with an error.
 * The values are checked by the Python tests; this one checks memory and
 * arithmetic hygiene, including the extremes (empty inputs, wrap-around). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

float orc_widen_bf16(uint16_t x);
void orc_aggregate_f32(const float *const *U, int K, int64_t n, const int32_t *order, int M,
                       const float *weights, float *out);
void orc_aggregate_bf16(const uint16_t *const *U, int K, int64_t n, const int32_t *order, int M,
                        const float *weights, float *out);
void orc_apply_ordered_f32(float *model, float *momentum, const float *const *U, int K, int64_t n,
                           const int32_t *order, int M, float lr, float mu);
void orc_apply_ordered_bf16(float *model, float *momentum, const uint16_t *const *U, int K,
                            int64_t n, const int32_t *order, int M, float lr, float mu);
void orc_aggregate_apply_f32(float *model, float *momentum, float *out, const float *const *U,
                             int K, int64_t n, const int32_t *order, int M, const float *weights,
                             float lr, float mu);
void orc_aggregate_apply_bf16(float *model, float *momentum, float *out, const uint16_t *const *U,
                              int K, int64_t n, const int32_t *order, int M, const float *weights,
                              float lr, float mu);
void orc_apply_grouped_f32(float *model, float *momentum, const float *const *U, int K, int64_t n,
                           const int32_t *order, int M, const float *weights,
                           const int32_t *group_len, int n_groups, float lr, float mu);
void orc_apply_grouped_bf16(float *model, float *momentum, const uint16_t *const *U, int K,
                            int64_t n, const int32_t *order, int M, const float *weights,
                            const int32_t *group_len, int n_groups, float lr, float mu);
double orc_sum_sq_f32(const float *x, int64_t n);
double orc_sum_sq_diff_f32(const float *a, const float *b, int64_t n);
double orc_sum_sq_bf16(const uint16_t *x, int64_t n);
double orc_divergence_bound(double h_norm, const double *g_norm, const float *wt, const int32_t *group_len,
                            int n_groups, double lr, double mu);
int64_t orc_scatter_add(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                        const int32_t *const *triples, const int64_t *n_triples, int K,
                        int32_t word_lo, int32_t word_hi, int32_t topic_lo, int32_t topic_hi,
                        int count_rejected);
void orc_counts_add_dense(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                          const int32_t *const *D, int K, int32_t word_lo, int32_t word_hi,
                          int32_t topic_lo, int32_t topic_hi);

static uint32_t state = 12345u;
static uint32_t next_u32(void)
{
    state = state * 1664525u + 1013904223u;
    return state;
}
static float next_float(void) { return (float)((int32_t)(next_u32() >> 8) - (1 << 23)) / (float)(1 << 20); }

static void *exact(size_t bytes) { return malloc(bytes ? bytes : 1); }

static void dense_calls(int K, int64_t n, int M)
{
    float **uf = exact(sizeof(float *) * (size_t)K);
    uint16_t **ub = exact(sizeof(uint16_t *) * (size_t)K);
    for (int k = 0; k < K; ++k) {
        uf[k] = exact(sizeof(float) * (size_t)n);
        ub[k] = exact(sizeof(uint16_t) * (size_t)n);
        for (int64_t i = 0; i < n; ++i) {
            uf[k][i] = next_float();
            ub[k][i] = (uint16_t)(next_u32() >> 16);
        }
    }
    int32_t *order = exact(sizeof(int32_t) * (size_t)M);
    for (int t = 0; t < M; ++t) order[t] = (K - 1 - t) % K;          /* a permutation prefix */
    float *weights = exact(sizeof(float) * (size_t)K);
    for (int k = 0; k < K; ++k) weights[k] = next_float();
    int32_t *lens = exact(sizeof(int32_t) * (size_t)(M ? M : 1));
    int n_groups = 0, left = M;
    while (left > 0) {
        int len = 1 + (int)(next_u32() % (uint32_t)left);
        lens[n_groups++] = len;
        left -= len;
    }
    float *w = exact(sizeof(float) * (size_t)n), *h = exact(sizeof(float) * (size_t)n);
    float *out = exact(sizeof(float) * (size_t)n);
    for (int64_t i = 0; i < n; ++i) {
        w[i] = next_float();
        h[i] = next_float();
    }
    const float *const *cuf = (const float *const *)uf;
    const uint16_t *const *cub = (const uint16_t *const *)ub;
    orc_aggregate_f32(cuf, K, n, order, M, weights, out);
    orc_aggregate_f32(cuf, K, n, order, M, NULL, out);
    orc_aggregate_bf16(cub, K, n, order, M, weights, out);
    orc_apply_ordered_f32(w, h, cuf, K, n, order, M, 0.1f, 0.9f);
    orc_apply_ordered_f32(w, NULL, cuf, K, n, order, M, 0.1f, 0.9f);
    orc_apply_ordered_bf16(w, h, cub, K, n, order, M, 0.1f, 0.9f);
    orc_aggregate_apply_f32(w, h, out, cuf, K, n, order, M, weights, 0.1f, 0.9f);
    orc_aggregate_apply_f32(w, NULL, NULL, cuf, K, n, order, M, NULL, 0.1f, 0.9f);
    orc_aggregate_apply_bf16(w, h, out, cub, K, n, order, M, weights, 0.1f, 0.9f);
    orc_apply_grouped_f32(w, h, cuf, K, n, order, M, weights, lens, n_groups, 0.1f, 0.9f);
    orc_apply_grouped_bf16(w, NULL, cub, K, n, order, M, NULL, lens, n_groups, 0.1f, 0.9f);
    volatile double sink = orc_sum_sq_f32(w, n) + orc_sum_sq_diff_f32(w, h, n) + orc_sum_sq_bf16(ub[0], n);
    double *g_norm = exact(sizeof(double) * (size_t)(M > 0 ? M : 1));
    for (int t = 0; t < M; ++t) g_norm[t] = 1.0 + t;
    /* (the weights of this driver are indexed by worker; any M of them will do here) */
    sink += orc_divergence_bound(2.0, g_norm, weights, lens, n_groups, 0.1, 0.9);
    sink += orc_divergence_bound(2.0, g_norm, NULL, lens, n_groups, 0.1, 0.9);
    (void)sink;
    free(g_norm);
    for (int k = 0; k < K; ++k) {
        free(uf[k]);
        free(ub[k]);
    }
    free(uf); free(ub); free(order); free(weights); free(lens); free(w); free(h); free(out);
}

static void sparse_calls(int32_t V, int32_t T, int K, int64_t m)
{
    size_t cells = (size_t)V * (size_t)T;
    int32_t *counts = exact(sizeof(int32_t) * cells), *totals = exact(sizeof(int32_t) * (size_t)T);
    for (size_t i = 0; i < cells; ++i) counts[i] = (int32_t)next_u32();       /* any value: sums wrap */
    for (int32_t t = 0; t < T; ++t) totals[t] = (int32_t)next_u32();
    int32_t **tr = exact(sizeof(int32_t *) * (size_t)K);
    int32_t **dense = exact(sizeof(int32_t *) * (size_t)K);
    int64_t *cnt = exact(sizeof(int64_t) * (size_t)K);
    for (int k = 0; k < K; ++k) {
        cnt[k] = k == 1 ? 0 : m;                                            /* one empty buffer */
        tr[k] = exact(sizeof(int32_t) * 3 * (size_t)cnt[k]);
        for (int64_t r = 0; r < cnt[k]; ++r) {
            tr[k][3 * r + 0] = (int32_t)(next_u32() % (uint32_t)(V + 2)) - 1;  /* -1 .. V: some invalid */
            tr[k][3 * r + 1] = (int32_t)(next_u32() % (uint32_t)(T + 2)) - 1;
            tr[k][3 * r + 2] = r % 7 == 0 ? INT32_MIN : (r % 5 == 0 ? INT32_MAX : (int32_t)next_u32());
        }
        dense[k] = exact(sizeof(int32_t) * cells);
        for (size_t i = 0; i < cells; ++i) dense[k][i] = (int32_t)next_u32();
    }
    const int32_t *const *ctr = (const int32_t *const *)tr;
    const int32_t *const *cd = (const int32_t *const *)dense;
    orc_scatter_add(counts, totals, V, T, ctr, cnt, K, 0, V, 0, T, 1);
    orc_scatter_add(counts, NULL, V, T, ctr, cnt, K, 0, V, 0, 0, 0);
    orc_scatter_add(counts, totals, V, T, ctr, cnt, K, V / 2, V, T / 2, T, 0);   /* a slice */
    orc_scatter_add(counts, totals, V, T, ctr, cnt, 0, 0, V, 0, T, 1);           /* no buffers */
    orc_counts_add_dense(counts, totals, V, T, cd, K, 0, V, 0, T);
    orc_counts_add_dense(counts, NULL, V, T, cd, K, 0, V, 0, 0);
    orc_counts_add_dense(counts, totals, V, T, cd, K, V / 2, V, T / 2, T);
    for (int k = 0; k < K; ++k) {
        free(tr[k]);
        free(dense[k]);
    }
    free(tr); free(dense); free(cnt); free(counts); free(totals);
}

int main(void)
{
    for (unsigned x = 0; x < 65536u; x += 257u) {
        volatile float f = orc_widen_bf16((uint16_t)x);
        (void)f;
    }
    dense_calls(1, 1, 1);
    dense_calls(3, 0, 2);          /* no elements */
    dense_calls(4, 17, 0);         /* empty order */
    dense_calls(5, 33, 5);
    dense_calls(64, 9, 40);
    sparse_calls(1, 1, 1, 10);
    sparse_calls(3, 2, 3, 50);
    sparse_calls(7, 5, 4, 1000);
    puts("oracle sanitizer run: ok");
    return 0;
}
