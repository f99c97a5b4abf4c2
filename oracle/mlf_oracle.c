/*
 * CPU oracle for the server-side hot path of MLfabric (arXiv 1907.00434).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the GPU
 * library is checked against.  Nothing in the product path may call it, and it
 * shares no source, header, table or helper with the GPU library.
 *
 * Precision: everything floating-point is IEEE binary32, round-to-nearest-even,
 * one rounding per written operation (build with -ffp-contract=off, no
 * fast-math, no flush-to-zero).  The paper states no precision; the required
 * parity bar is bit-exactness in binary32, so the oracle works in binary32 and
 * is itself pinned against exact rational / binary64 evaluations in the tests.
 *
 * Every loop below works on a half-open element range handed in as
 * (pointer, n); a caller may split [0,n) into slices and call once per slice,
 * because no element's result depends on any other element.
 *
 * What is computed, and where the paper defines it:
 *
 *  - orc_aggregate_*       Sec. 4 "Architecture": an aggregator computes the
 *                          (weighted) sum of the updates routed to it; Sec. 3.2
 *                          four-worker example r = g3 + g4; Sec. 5.2: the order
 *                          chosen by the scheduler is preserved through the
 *                          aggregator.  The sum is taken left to right in the
 *                          scheduler's order.
 *  - orc_apply_ordered_*   Eq. 2 (server model update with momentum),
 *                          w_{t+1} = w_t + u_t + gamma (w_t - w_{t-1}), applied
 *                          once per update in the given order, with u = -eta g
 *                          (Eq. 1 without its regulariser) and the history
 *                          h = w_t - w_{t-1} (Sec. 3.3, definition of h^0) kept
 *                          in the momentum buffer:  h <- gamma h - eta g ;
 *                          w <- w + h.
 *  - orc_aggregate_apply_* Sec. 5.4 "Synchronous SGD/PS": the updates of one
 *                          iteration are aggregated and the aggregate is applied
 *                          to the model once (one step of Eq. 2 with g = sum).
 *  - orc_apply_grouped_*   Sec. 5.2 "Aggregation": a batch reaches the server as a
 *                          directly forwarded prefix followed by groups that
 *                          were summed at aggregators; each arrival is one step
 *                          of Eq. 2.
 *  - orc_sum_sq_*          Table 1 (push carries update_norm) and Sec. 5.3
 *                          (divergence bound from ||h||, ||u_i||; exact
 *                          divergence ||w_s - w_r||): squared 2-norms.
 *  - orc_divergence_bound  Sec. 5.3: the upper bound of a batch's divergence
 *                          that the scheduler forms from those norms.
 *  - orc_counts_add_dense  Sec. 6: the same LDA update exchanged as dense V x T
 *                          delta matrices, summed over the workers.
 *  - orc_scatter_add       Sec. 6 "Datasets and ML models": an LDA worker's
 *                          update is a numerical update to the word-topic count
 *                          matrix; here it arrives as (word, topic, delta)
 *                          triples that are added into the matrix and into the
 *                          per-topic totals.
 */
#include <stddef.h>
#include <math.h>
#include <stdint.h>
#include <string.h>

/* bfloat16 -> binary32: the 16 stored bits are the top half of the float. */
static float widen_bf16(uint16_t x)
{
    uint32_t bits = (uint32_t)x << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return f;
}

float orc_widen_bf16(uint16_t x) { return widen_bf16(x); }

/* ------------------------------------------------------------------------ */
/* Weighted, ordered sum of M of the K update vectors (Sec. 4; Sec. 5.2).     */
/*   out[i] = sum_{t=0}^{M-1} weights[order[t]] * U[order[t]][i]              */
/* summed left to right.  The accumulator starts as the first term (no        */
/* leading "0 +"), so M = 1 with no weights is a bit copy and -0 survives.    */
/* weights == NULL means every weight is 1 and no multiply is performed.      */
/* M == 0 gives +0.                                                           */
/* ------------------------------------------------------------------------ */
static float ordered_sum_f32(const float *const *U, int64_t i,
                             const int32_t *order, int M, const float *weights)
{
    float acc = 0.0f;
    for (int t = 0; t < M; ++t) {
        int j = order[t];
        float term = U[j][i];
        if (weights) {
            term = weights[j] * term;
        }
        if (t == 0) {
            acc = term;
        } else {
            acc = acc + term;
        }
    }
    return acc;
}

static float ordered_sum_bf16(const uint16_t *const *U, int64_t i,
                              const int32_t *order, int M, const float *weights)
{
    float acc = 0.0f;
    for (int t = 0; t < M; ++t) {
        int j = order[t];
        float term = widen_bf16(U[j][i]);
        if (weights) {
            term = weights[j] * term;
        }
        if (t == 0) {
            acc = term;
        } else {
            acc = acc + term;
        }
    }
    return acc;
}

void orc_aggregate_f32(const float *const *U, int K, int64_t n,
                       const int32_t *order, int M, const float *weights,
                       float *out)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        out[i] = ordered_sum_f32(U, i, order, M, weights);
    }
}

void orc_aggregate_bf16(const uint16_t *const *U, int K, int64_t n,
                        const int32_t *order, int M, const float *weights,
                        float *out)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        out[i] = ordered_sum_bf16(U, i, order, M, weights);
    }
}

/* ------------------------------------------------------------------------ */
/* One application of Eq. 2 with u = -lr * g.                                 */
/* With a history buffer:   h <- mu*h - lr*g ;  w <- w + h                    */
/* (two products, one difference, one sum: four roundings).                   */
/* Without one (plain SGD):  w <- w - lr*g.                                    */
/* ------------------------------------------------------------------------ */
static void server_step(float *w, float *h, int have_h, float g, float lr,
                        float mu)
{
    float q = lr * g;
    if (have_h) {
        float p = mu * (*h);
        float hn = p - q;
        *h = hn;
        *w = *w + hn;
    } else {
        *w = *w - q;
    }
}

/* Eq. 2 folded over the scheduler's sequence, one update after another. */
void orc_apply_ordered_f32(float *model, float *momentum,
                           const float *const *U, int K, int64_t n,
                           const int32_t *order, int M, float lr, float mu)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        for (int t = 0; t < M; ++t) {
            server_step(&w, &h, momentum != NULL, U[order[t]][i], lr, mu);
        }
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

void orc_apply_ordered_bf16(float *model, float *momentum,
                            const uint16_t *const *U, int K, int64_t n,
                            const int32_t *order, int M, float lr, float mu)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        for (int t = 0; t < M; ++t) {
            server_step(&w, &h, momentum != NULL,
                        widen_bf16(U[order[t]][i]), lr, mu);
        }
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Synchronous iteration (Sec. 5.4): aggregate, then ONE step of Eq. 2 with   */
/* g = the aggregate.  out (optional) receives the aggregate.                 */
/* ------------------------------------------------------------------------ */
void orc_aggregate_apply_f32(float *model, float *momentum, float *out,
                             const float *const *U, int K, int64_t n,
                             const int32_t *order, int M, const float *weights,
                             float lr, float mu)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        float a = ordered_sum_f32(U, i, order, M, weights);
        if (out) {
            out[i] = a;
        }
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        server_step(&w, &h, momentum != NULL, a, lr, mu);
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

void orc_aggregate_apply_bf16(float *model, float *momentum, float *out,
                              const uint16_t *const *U, int K, int64_t n,
                              const int32_t *order, int M, const float *weights,
                              float lr, float mu)
{
    (void)K;
    for (int64_t i = 0; i < n; ++i) {
        float a = ordered_sum_bf16(U, i, order, M, weights);
        if (out) {
            out[i] = a;
        }
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        server_step(&w, &h, momentum != NULL, a, lr, mu);
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* One scheduled batch as it reaches the server (Sec. 5.2 "Aggregation"): the  */
/* ordered updates are cut into consecutive groups; the first group goes to    */
/* the server directly (every update applied on its own: groups of length 1),  */
/* each later group is summed at an aggregator and arrives as ONE update.      */
/* Group j covers the next group_len[j] entries of `order`; for each group, in */
/* sequence:  a = ordered weighted sum of the group ; one step of Eq. 2 with   */
/* g = a.  The lengths are positive and add up to M.                           */
/* ------------------------------------------------------------------------ */
void orc_apply_grouped_f32(float *model, float *momentum, const float *const *U,
                           int K, int64_t n, const int32_t *order, int M,
                           const float *weights, const int32_t *group_len,
                           int n_groups, float lr, float mu)
{
    (void)K;
    (void)M;
    for (int64_t i = 0; i < n; ++i) {
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        int first = 0;
        for (int j = 0; j < n_groups; ++j) {
            float a = ordered_sum_f32(U, i, order + first, group_len[j], weights);
            server_step(&w, &h, momentum != NULL, a, lr, mu);
            first += group_len[j];
        }
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

void orc_apply_grouped_bf16(float *model, float *momentum,
                            const uint16_t *const *U, int K, int64_t n,
                            const int32_t *order, int M, const float *weights,
                            const int32_t *group_len, int n_groups, float lr,
                            float mu)
{
    (void)K;
    (void)M;
    for (int64_t i = 0; i < n; ++i) {
        float w = model[i];
        float h = momentum ? momentum[i] : 0.0f;
        int first = 0;
        for (int j = 0; j < n_groups; ++j) {
            float a = ordered_sum_bf16(U, i, order + first, group_len[j], weights);
            server_step(&w, &h, momentum != NULL, a, lr, mu);
            first += group_len[j];
        }
        model[i] = w;
        if (momentum) {
            momentum[i] = h;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Squared Euclidean norms (Table 1: a push carries update_norm; Sec. 5.3: the */
/* divergence bound is built from ||h|| and ||u_i||, and the exact divergence   */
/* is ||w_s - w_r||_2).  Squares of binary32 values and their differences are  */
/* exact in binary128, and the running sum is kept in binary128, so the value  */
/* returned is the true sum rounded (up to 2^-100 or so) to binary64.          */
/* ------------------------------------------------------------------------ */
double orc_sum_sq_f32(const float *x, int64_t n)
{
    __float128 acc = 0;
    for (int64_t i = 0; i < n; ++i) {
        __float128 v = x[i];
        acc += v * v;
    }
    return (double)acc;
}

double orc_sum_sq_diff_f32(const float *a, const float *b, int64_t n)
{
    __float128 acc = 0;
    for (int64_t i = 0; i < n; ++i) {
        __float128 d = (__float128)a[i] - (__float128)b[i];
        acc += d * d;
    }
    return (double)acc;
}

/* The same for an update that arrives in bfloat16: every element is widened   */
/* exactly, as the aggregation does, before it is squared.                     */
double orc_sum_sq_bf16(const uint16_t *x, int64_t n)
{
    __float128 acc = 0;
    for (int64_t i = 0; i < n; ++i) {
        __float128 v = widen_bf16(x[i]);
        acc += v * v;
    }
    return (double)acc;
}

/* ------------------------------------------------------------------------ */
/* Upper bound of the divergence a batch causes (Sec. 5.3: the scheduler does   */
/* not compute ||w_after - w_before||_2, it bounds it from the norms of the     */
/* history and of the updates).  The batch is n_groups server steps of Eq. 2;   */
/* step j applies u_j = -lr * (sum over the group's updates of wt * g).         */
/* Unrolling Eq. 2 over the steps (the two-step case is printed in Sec. 3.3:    */
/* (mu + mu^2) h0 + (1 + mu) u_1 + u_2):                                        */
/*   w_after - w_before = (mu + ... + mu^S) h0                                  */
/*                        + sum_j (1 + mu + ... + mu^(S-j)) u_j ,  j = 1..S     */
/* and by the triangle inequality, for the norm of the whole and of each u_j,   */
/*   bound = (mu + ... + mu^S) ||h0|| + sum_j (1 + ... + mu^(S-j)) ||u_j||,     */
/*   ||u_j|| <= lr * sum over the group of |wt| * ||g||.                        */
/* Its square is the printed form a1 ||h0||^2 + a2 ||u1||^2 + ... with every    */
/* cross term taken at its Cauchy-Schwarz maximum.  g_norm[t] and wt[t] belong  */
/* to the t-th committed update (wt NULL = 1); the groups tile the sequence.    */
/* ------------------------------------------------------------------------ */
double orc_divergence_bound(double h_norm, const double *g_norm, const float *wt,
                            const int32_t *group_len, int n_groups, double lr, double mu)
{
    double bound = 0.0;
    double geometric = 0.0;                 /* mu + mu^2 + ... + mu^S */
    double power = 1.0;
    for (int j = 0; j < n_groups; ++j) {
        power *= mu;
        geometric += power;
    }
    bound += fabs(geometric) * h_norm;
    int t = 0;
    for (int j = 0; j < n_groups; ++j) {
        double u_norm = 0.0;                /* bound of ||u_j|| */
        for (int i = 0; i < group_len[j]; ++i, ++t) {
            u_norm += fabs(wt != 0 ? (double)wt[t] : 1.0) * g_norm[t];
        }
        u_norm *= fabs(lr);
        double coefficient = 0.0;           /* 1 + mu + ... + mu^(S-1-j) */
        double p = 1.0;
        for (int i = j; i < n_groups; ++i) {
            coefficient += p;
            p *= mu;
        }
        bound += fabs(coefficient) * u_norm;
    }
    return bound;
}

/* ------------------------------------------------------------------------ */
/* LDA count deltas (Sec. 6): for every (word, topic, delta) triple            */
/*   counts[word*T + topic] += delta ;  totals[topic] += delta                */
/* Additions wrap modulo 2^32 (done on unsigned values so that C defines it). */
/* A triple whose word or topic is out of range is skipped and counted.       */
/*                                                                            */
/* The caller may restrict which part of the state this call owns: counts     */
/* rows in [word_lo, word_hi) and totals entries in [topic_lo, topic_hi) are   */
/* updated, the rest is left alone; rejected triples are counted only when    */
/* count_rejected is non-zero.  The full operation is one call with           */
/* (0, V, 0, T, 1); slices that partition both ranges give the same state.    */
/* Returns the number of rejected triples it counted.                         */
/* ------------------------------------------------------------------------ */
int64_t orc_scatter_add(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                        const int32_t *const *triples, const int64_t *n_triples,
                        int K, int32_t word_lo, int32_t word_hi,
                        int32_t topic_lo, int32_t topic_hi, int count_rejected)
{
    int64_t rejected = 0;
    for (int k = 0; k < K; ++k) {
        const int32_t *tr = triples[k];
        for (int64_t r = 0; r < n_triples[k]; ++r) {
            int32_t word = tr[3 * r + 0];
            int32_t topic = tr[3 * r + 1];
            int32_t delta = tr[3 * r + 2];
            if (word < 0 || word >= V || topic < 0 || topic >= T) {
                if (count_rejected) {
                    ++rejected;
                }
                continue;
            }
            if (word >= word_lo && word < word_hi) {
                int64_t cell = (int64_t)word * T + topic;
                counts[cell] =
                    (int32_t)((uint32_t)counts[cell] + (uint32_t)delta);
            }
            if (totals && topic >= topic_lo && topic < topic_hi) {
                totals[topic] =
                    (int32_t)((uint32_t)totals[topic] + (uint32_t)delta);
            }
        }
    }
    return rejected;
}

/* ------------------------------------------------------------------------ */
/* LDA update exchanged as a dense matrix (Sec. 6: every worker computes a      */
/* numerical update to the whole word-topic matrix and the updates are summed, */
/* as gradient updates are).  D[k] is worker k's V x T int32 delta matrix:     */
/*   counts[w*T + t] += sum_k D[k][w*T + t] ;  totals[t] += sum_w sum_k D[k][w*T + t] */
/* with wrap-around modulo 2^32.  A call owns the counts rows in               */
/* [word_lo, word_hi) and the totals entries in [topic_lo, topic_hi).          */
/* ------------------------------------------------------------------------ */
void orc_counts_add_dense(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                          const int32_t *const *D, int K, int32_t word_lo,
                          int32_t word_hi, int32_t topic_lo, int32_t topic_hi)
{
    for (int64_t w = word_lo; w < word_hi; ++w) {
        for (int64_t t = 0; t < T; ++t) {
            uint32_t s = 0;
            for (int k = 0; k < K; ++k) {
                s += (uint32_t)D[k][w * T + t];
            }
            counts[w * T + t] = (int32_t)((uint32_t)counts[w * T + t] + s);
        }
    }
    if (totals) {
        for (int64_t t = topic_lo; t < topic_hi; ++t) {
            uint32_t s = 0;
            for (int64_t w = 0; w < V; ++w) {
                for (int k = 0; k < K; ++k) {
                    s += (uint32_t)D[k][w * T + t];
                }
            }
            totals[t] = (int32_t)((uint32_t)totals[t] + s);
        }
    }
}
