/*
 * mlfabric.h -- C ABI of the MI355X (gfx950) library for the server-side hot
 * path of MLfabric (arXiv 1907.00434): the K-way reduction of worker update
 * vectors in the scheduler's order, the application of the aggregate or of the
 * ordered update sequence to the model, and the scatter-add of LDA count deltas.
 *
 * Common conventions
 * ------------------
 *  - "host" arguments (pointer tables, order, weights, triple counts) describe
 *    the scheduler's decisions.  They are read before the call returns and may
 *    be freed or changed right after it.
 *  - "device" arguments are HIP device pointers owned by the caller.  The
 *    library allocates no memory and frees nothing; the only state it keeps
 *    between calls is the scratch array of mlf_divergence_static (below).
 *    Device buffers must stay valid until the stream has run the enqueued work.
 *  - Every call only enqueues kernels on `stream` (a hipStream_t; NULL is the
 *    default stream) and returns; it never synchronises the device.
 *  - Errors are reported through the return code only; nothing is enqueued when
 *    a call returns an error other than MLF_EHIP.
 *  - Dense vectors: n contiguous elements.  Updates are MLF_F32 (IEEE binary32)
 *    or MLF_BF16 (bfloat16, widened exactly to binary32 before any arithmetic).
 *    model, momentum and out are always binary32.  Pointers must be aligned to
 *    their element size (else MLF_EALIGN); when every pointer of a call is
 *    16-byte aligned the 128-bit path is taken, otherwise a slower
 *    element-wise path gives the same bits.
 *  - Arithmetic is binary32, round-to-nearest-even, one rounding per operation
 *    written below (no fused multiply-add), subnormals kept.  For a fixed
 *    `order` the result is reproducible bit for bit.
 *  - `order` lists n_order <= K distinct worker indices in [0, K): the sequence
 *    in which the scheduler committed the updates (Sec. 5.1-5.2 of the paper).
 *    Workers that are not listed were dropped by the scheduler (Sec. 5.1,
 *    deadline / look-ahead drops) and are ignored; their pointers may be NULL.
 *  - model / momentum / out must not overlap each other or any listed update
 *    (MLF_EINVAL).
 */
#ifndef MLFABRIC_H
#define MLFABRIC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MLF_OK = 0,
    MLF_EINVAL = -1,        /* bad argument (see each call)                    */
    MLF_EALIGN = -2,        /* a device pointer is not aligned to its element  */
    MLF_EUNSUPPORTED = -3,  /* K > MLF_MAX_K, or n > MLF_STATIC_MAX_N          */
    MLF_EHIP = -4,          /* the HIP runtime refused the launch              */
    MLF_STATUS_INT32 = 0x7fffffff   /* not a status: makes every int a valid value of the type */
} mlf_status;

typedef enum { MLF_F32 = 0, MLF_BF16 = 1 } mlf_dtype;

typedef void *mlf_stream;   /* a hipStream_t */

#define MLF_MAX_K 64        /* most updates (or triple buffers) per call */
#define MLF_STATIC_MAX_N (1ll << 28)   /* most elements mlf_divergence_static takes */

/*
 * Aggregator (Sec. 4 "Architecture": aggregators compute the (weighted) sum of
 * incoming updates; Sec. 3.2 example r = g3 + g4; Sec. 5.2: the scheduler's
 * order is kept through the aggregator).
 *
 *   out[i] = sum_{t=0}^{n_order-1} weights[order[t]] * U_{order[t]}[i]
 *
 * summed left to right in that order; each product is rounded, then each sum.
 * The first term starts the accumulator (no "0 +").  weights == NULL means all
 * weights are 1 (multiplying by 1 is exact, so the result is the plain ordered
 * sum).  n_order == 0 writes +0 everywhere; n == 0 does nothing.
 *
 *   update_ptrs  host   K device pointers, one vector of n elements per worker
 *   order        host   n_order indices (may be NULL when n_order == 0)
 *   weights      host   K floats indexed by worker, or NULL
 *   out          device binary32[n]
 *
 * MLF_EINVAL: K < 1, n < 0, n_order outside [0, K], an index outside [0, K) or
 * listed twice, NULL out / update_ptrs / a listed update, overlap.
 */
mlf_status mlf_aggregate(const void *const *update_ptrs, int K, int64_t n,
                         mlf_dtype dtype, const int32_t *order, int n_order,
                         const float *weights, float *out, mlf_stream stream);

/*
 * Server update callback (Eq. 2 of the paper, SGD with momentum)
 *   w_{t+1} = w_t + u_t + gamma (w_t - w_{t-1}),   u = -lr * g  (Eq. 1),
 * applied once per listed update, in order, in ONE pass over the model.  The
 * momentum buffer holds the history h = w_t - w_{t-1} (Sec. 3.3, h^0).  For
 * each element and each t = 0 .. n_order-1:
 *
 *   p = mu * h ;  q = lr * g_{order[t]} ;  h = p - q ;  w = w + h
 *
 * momentum == NULL selects plain SGD (mu is ignored):  q = lr * g ; w = w - q.
 * Note that h is the paper's history, not the velocity of the v <- mu v + g
 * formulation; for constant lr the two give the same trajectory with
 * h = -lr v but round differently.
 *
 *   model     device binary32[n], read and written
 *   momentum  device binary32[n], read and written, or NULL
 *   others    as for mlf_aggregate
 *
 * n_order == 0 or n == 0 does nothing.  MLF_EINVAL as for mlf_aggregate
 * (model in place of out).
 */
mlf_status mlf_apply_ordered(float *model, float *momentum,
                             const void *const *update_ptrs, int K, int64_t n,
                             mlf_dtype dtype, const int32_t *order, int n_order,
                             float lr, float mu, mlf_stream stream);

/*
 * Synchronous iteration (Sec. 5.4 "Synchronous SGD/PS": the updates of an
 * iteration are aggregated and applied to the model): the sum of
 * mlf_aggregate, kept in registers, followed by ONE step of mlf_apply_ordered
 * with g = that sum.  Bit-identical to calling mlf_aggregate and then
 * mlf_apply_ordered on its output.  out_or_null (device binary32[n]) also
 * receives the aggregate when given.  n_order == 0 takes the step with g = +0
 * (the momentum term still moves the model).
 */
mlf_status mlf_aggregate_apply(float *model, float *momentum, float *out_or_null,
                               const void *const *update_ptrs, int K, int64_t n,
                               mlf_dtype dtype, const int32_t *order, int n_order,
                               const float *weights, float lr, float mu,
                               mlf_stream stream);

/*
 * One scheduled batch as it reaches the server (Sec. 5.2 "Aggregation" and
 * Alg. 3: the ordered updates are cut into consecutive groups; the first group
 * is forwarded to the server directly, every later group is summed at an
 * aggregator and arrives as one update; the order is kept throughout).  Group j
 * covers the next group_len[j] entries of `order`.  For each group, in sequence,
 *
 *   a = sum over the group of weights[order[t]] * U_{order[t]}   (as mlf_aggregate)
 *   p = mu * h ;  q = lr * a ;  h = p - q ;  w = w + h            (as mlf_apply_ordered)
 *
 * all in ONE pass over model and momentum and with every update read once; no
 * aggregate is written to memory.  A directly forwarded update is a group of
 * length 1.  Bit-identical to calling mlf_aggregate per group and then
 * mlf_apply_ordered over the aggregates.  All groups of length 1 without weights
 * is mlf_apply_ordered; a single group is mlf_aggregate_apply.
 *
 *   group_len  host  n_groups positive lengths that add up to n_order
 *   others     as for mlf_aggregate / mlf_apply_ordered
 *
 * MLF_EINVAL additionally for a length < 1 or lengths that do not add up to
 * n_order.  n_order == 0 (with n_groups == 0) or n == 0 does nothing.
 */
mlf_status mlf_apply_grouped(float *model, float *momentum,
                             const void *const *update_ptrs, int K, int64_t n,
                             mlf_dtype dtype, const int32_t *order, int n_order,
                             const float *weights, const int32_t *group_len,
                             int n_groups, float lr, float mu, mlf_stream stream);

/*
 * Norms for the scheduler, fused into the passes above at no extra HBM traffic.
 * A push carries the update's norm (Table 1, push(server, update, update_norm)),
 * and the scheduler bounds the server-replica divergence from ||h|| and the
 * ||u_i|| alone because the exact divergence ||w_s - w_r||_2 is costly to
 * compute (Sec. 5.3); here both come out of the pass that is made anyway.
 *
 * mlf_aggregate_norm: mlf_aggregate, and norm_sq[0] = sum_i out[i]^2 -- the
 * squared norm of the aggregate an aggregator forwards.
 *
 * mlf_apply_grouped_norms: mlf_apply_grouped, and
 *   norms_sq[0] = sum_i h[i]^2 of the history after the call (0 without momentum)
 *   norms_sq[1] = sum_i (w_after[i] - w_before[i])^2: the exact squared divergence
 *                 between the server after this batch and a replica that has not
 *                 applied it yet.
 * With n_order == 0 the model is left as it is and the norms describe it.
 *
 * The sums are taken in binary64 (squares of binary32 values are exact there; a
 * difference w_after - w_before is rounded once to binary64) in a fixed order,
 * so a call repeated with the same arguments on the same device gives the same
 * bits.  The order depends on n, on the data type of the updates, on whether
 * every pointer of the call is 16-byte aligned (128-bit or element-wise path),
 * on whether momentum is given, whether 4n bytes per written vector exceed
 * 256 MiB in total and, if so, whether 8 or more updates (4 or more for the
 * aggregate, 16 or more for the update-norm variants below) are committed
 * (these select the tile shape), and on the number of XCDs of the device; calls
 * that differ in any of these may differ in the last bits.
 * The sums agree with the exactly rounded ones to about 1e-14 relative.
 *
 *   norm_sq / norms_sq  device, 1 / 2 doubles, 8-byte aligned; written
 *   workspace           device scratch of mlf_norms_workspace_bytes(n) bytes,
 *                       16-byte aligned (MLF_EINVAL if NULL or too small)
 */
size_t mlf_norms_workspace_bytes(int64_t n);

mlf_status mlf_aggregate_norm(const void *const *update_ptrs, int K, int64_t n,
                              mlf_dtype dtype, const int32_t *order, int n_order,
                              const float *weights, float *out, double *norm_sq,
                              void *workspace, size_t workspace_bytes,
                              mlf_stream stream);

mlf_status mlf_apply_grouped_norms(float *model, float *momentum,
                                   const void *const *update_ptrs, int K, int64_t n,
                                   mlf_dtype dtype, const int32_t *order, int n_order,
                                   const float *weights, const int32_t *group_len,
                                   int n_groups, float lr, float mu, double *norms_sq,
                                   void *workspace, size_t workspace_bytes,
                                   mlf_stream stream);

/*
 * The same two calls with the squared norm of every committed update as well
 * (Table 1: a push carries update_norm; Sec. 5.3: the scheduler bounds the
 * divergence from ||h|| and the ||u_i||).  The server or aggregator reads every
 * update anyway, so the norms cost no further HBM traffic:
 *
 *   update_norm_sq[t] = sum_i U_order[t][i]^2,   t = 0 .. n_order - 1
 *
 * of the update as it arrived (before its weight; bfloat16 widened exactly), in
 * the commit sequence.  norm_sq / norms_sq are as in the calls above.  Sums in
 * binary64 in a fixed order (exact squares, rounded additions): repeatable bit
 * for bit for the same arguments on the same device; the order depends on what
 * the calls above list and on the number of compute units of the device and
 * the size of their LDS, and a
 * sum agrees with the exactly rounded one to about 1e-14 relative.  These
 * variants keep one running sum per update and lane on chip (binary64
 * arithmetic per update element) and walk the vector with a fixed number of
 * workgroups, which makes the pass itself 7 to 20 per cent slower than
 * mlf_aggregate_norm / mlf_apply_grouped_norms.
 *
 *   update_norm_sq  device, n_order doubles, 8-byte aligned; written
 *   workspace       device scratch of mlf_update_norms_workspace_bytes(n) bytes
 *                   (about 6.5 MiB whatever n), 16-byte aligned
 */
size_t mlf_update_norms_workspace_bytes(int64_t n);

mlf_status mlf_aggregate_update_norms(const void *const *update_ptrs, int K, int64_t n,
                                      mlf_dtype dtype, const int32_t *order, int n_order,
                                      const float *weights, float *out, double *norm_sq,
                                      double *update_norm_sq, void *workspace,
                                      size_t workspace_bytes, mlf_stream stream);

mlf_status mlf_apply_grouped_update_norms(float *model, float *momentum,
                                          const void *const *update_ptrs, int K, int64_t n,
                                          mlf_dtype dtype, const int32_t *order, int n_order,
                                          const float *weights, const int32_t *group_len,
                                          int n_groups, float lr, float mu, double *norms_sq,
                                          double *update_norm_sq, void *workspace,
                                          size_t workspace_bytes, mlf_stream stream);

/*
 * The scheduler's upper bound of the divergence a batch will cause (Sec. 5.3:
 * ||w_s - w_r||_2 is approximated from above with the norms of the history and
 * of the updates, and a schedule is admissible if the bound stays below
 * Div_max).  For a batch applied as n_groups server steps of Eq. 2 (the shape
 * mlf_apply_grouped takes; single updates are groups of length 1), unrolling
 * Eq. 2 gives
 *
 *   w_after - w_before = (mu + ... + mu^S) h0 + sum_j (1 + mu + ... + mu^(S-j)) u_j
 *   u_j = -lr * sum over group j of weights * g            (S = n_groups, j = 1..S)
 *
 * (the two-update case printed in Sec. 3.3 is (mu + mu^2) h0 + (1 + mu) u_1 + u_2)
 * and the triangle inequality on the whole and on every u_j gives
 *
 *   bound = |mu + ... + mu^S| ||h0|| + |lr| sum_j |1 + ... + mu^(S-j)| sum_group |weight| ||g||.
 *
 * Its square is the paper's a1 ||h0||^2 + a2 ||u1||^2 + ... with every cross term
 * at its Cauchy-Schwarz maximum (the printed list of cross terms names one
 * product twice and omits another, and gives no constants).  The exact value,
 * for comparison, is what mlf_apply_grouped_norms returns in norms_sq[1].
 * Host arithmetic only, no GPU work; all pointers are host pointers.
 *
 *   h_norm_sq       ||h0||^2 of the history before the batch (0 without momentum)
 *   update_norm_sq  n_order squared norms in the commit sequence, as
 *                   mlf_*_update_norms return them
 *   order, weights  as in mlf_apply_grouped (weights indexed by worker, NULL = 1)
 *   bound           one double; written: an upper bound of ||w_after - w_before||_2
 *
 * MLF_EINVAL: NULL bound, K < 1, n_order outside [0, K], an index outside
 * [0, K), groups that do not tile the sequence, a negative or NaN norm.
 * MLF_EUNSUPPORTED: K > MLF_MAX_K.
 */
mlf_status mlf_divergence_bound(double h_norm_sq, const double *update_norm_sq,
                                const int32_t *order, int n_order, int K,
                                const float *weights, const int32_t *group_len,
                                int n_groups, float lr, float mu, double *bound);

/*
 * Exact server-replica divergence (Sec. 3.3 "Enforcing bounded consistency" and
 * Sec. 5.3: the replica is kept within ||w_s - w_r||_2 <= Div_max of the server).
 *   dist_sq[0] = sum_i (w_server[i] - w_replica[i])^2
 * in binary64, each difference rounded once, summed in an order fixed by n and
 * by whether both vectors are 16-byte aligned, so reproducible bit for bit.  A replica catches up by applying the updates it
 * lags by with mlf_apply_ordered / mlf_apply_grouped in the server's order; the
 * same updates in the same order give the same model bit for bit.
 *
 *   w_server, w_replica  device binary32[n], read only, may be the same vector
 *   dist_sq              device, 1 double, 8-byte aligned; written
 *   workspace            device scratch of mlf_norms_workspace_bytes(n) bytes,
 *                        16-byte aligned
 */
mlf_status mlf_divergence(const float *w_server, const float *w_replica, int64_t n,
                          double *dist_sq, void *workspace, size_t workspace_bytes,
                          mlf_stream stream);

/*
 * mlf_divergence for callers that cannot allocate device memory and so have no
 * workspace to pass: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace, same
 * kernels, same result bit for bit.  The partial sums go to an array of 12,352
 * pairs of doubles (197,632 bytes) that is part of the
 * library's device code: every GPU the library runs on holds one copy until the
 * process ends.  The call allocates and frees nothing; the first call on a
 * device looks up the address of that device's copy (make it outside a graph
 * capture) and later calls reuse it.
 *
 * All calls on one GPU share that array: two calls whose work may overlap on the
 * device (different streams, or graph branches that run side by side) race and
 * give wrong distances; order them on one stream or with events.  The array
 * keeps the previous call's partial sums; every entry a call reads it has
 * written first, so nothing needs clearing.
 *
 * MLF_EUNSUPPORTED: n > MLF_STATIC_MAX_N (use mlf_divergence with a workspace),
 * or a device ordinal above 63.  Otherwise as mlf_divergence.
 */
mlf_status mlf_divergence_static(const float *w_server, const float *w_replica, int64_t n,
                                 double *dist_sq, mlf_stream stream);

/*
 * LDA count deltas (Sec. 6 "Datasets and ML models": each LDA worker computes a
 * numerical update to the word-topic matrix).  For every triple
 * (word, topic, delta) of every buffer:
 *
 *   counts[word * T + topic] += delta ;  totals[topic] += delta
 *
 * in int32 arithmetic that wraps modulo 2^32.  Integer addition commutes, so
 * the result does not depend on execution order.  A triple with word outside
 * [0, V) or topic outside [0, T) is skipped and counted in *n_rejected.
 *
 *   counts        device int32[V*T], row-major by word; read and written
 *   totals        device int32[T] or NULL
 *   triple_ptrs   host   K device pointers; buffer k holds n_triples[k] triples
 *                        as 3 consecutive int32 (word, topic, delta), 4-byte
 *                        aligned
 *   n_triples     host   K counts (>= 0)
 *   workspace     device scratch of at least
 *                        mlf_sparse_workspace_bytes(V, T, total) bytes, 256-byte
 *                        aligned, contents undefined before and after.  With it
 *                        the triples are first grouped by the 128 KiB tile of
 *                        counts[] they hit (several times faster for large
 *                        batches); the groups are laid out from a sample of the
 *                        triples (of every buffer, every p-th block of 256
 *                        consecutive triples, p = total / (256 * tiles) kept
 *                        within [1, 64], tiles = ceil(V*T / 32768)), and a
 *                        triple that finds its group full is added directly,
 *                        so the result never depends on the sample; a batch
 *                        whose sampled blocks say nothing about the others
 *                        runs at the direct path's speed.  With NULL (or fewer
 *                        bytes, or a shape that
 *                        path does not serve) the call takes the direct path,
 *                        which needs none and gives the same result
 *   n_rejected    device int32 counter that the call ADDS to (the caller clears
 *                        it), or NULL
 *
 * MLF_EINVAL: V < 1, T < 1, K < 0, a negative count, a NULL buffer with a
 * positive count, NULL counts.  K == 0 or no triples does nothing.
 * MLF_EUNSUPPORTED: K > MLF_MAX_K.  The triple buffers must not change between
 * the call and the completion of its work on the stream.
 */
mlf_status mlf_sparse_scatter_add(int32_t *counts, int32_t *totals, int32_t V,
                                  int32_t T, const int32_t *const *triple_ptrs,
                                  const int64_t *n_triples, int K,
                                  void *workspace, size_t workspace_bytes,
                                  int32_t *n_rejected, mlf_stream stream);

/* Scratch the grouped path of mlf_sparse_scatter_add needs for this problem
 * size: 8 to 14 bytes per triple.  0 when that path would not be used: a
 * matrix of more than 2^30 cells, or a batch so small that the direct path is
 * faster (fewer than 262,144 + 600 per 32,768 cells of the matrix triples). */
size_t mlf_sparse_workspace_bytes(int32_t V, int32_t T, int64_t total_triples);

/*
 * The same LDA update exchanged as dense matrices (Sec. 6: every worker computes
 * a numerical update to the whole word-topic matrix, and the updates are
 * exchanged and summed like gradient updates):
 *
 *   counts[c] += sum_k delta_k[c]   for every cell c of the V x T matrix
 *   totals[t] += sum_w sum_k delta_k[w*T + t]
 *
 * in int32 arithmetic that wraps modulo 2^32 (order-free).  Every delta matrix
 * is read once, counts is read and written once.
 *
 *   counts      device int32[V*T], row-major; read and written
 *   totals      device int32[T] or NULL
 *   delta_ptrs  host   K device pointers to int32[V*T] matrices, 4-byte aligned
 *                      (16-byte alignment of all pointers selects 128-bit loads)
 *
 * MLF_EINVAL: NULL counts / table / matrix, V < 1, T < 1, K < 0, a delta matrix
 * overlapping counts.  K == 0 does nothing.  MLF_EUNSUPPORTED: K > MLF_MAX_K.
 */
mlf_status mlf_counts_add_dense(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                                const int32_t *const *delta_ptrs, int K,
                                mlf_stream stream);

/* Static, human-readable name of a status code; any other value gives
 * "unknown mlf_status". */
const char *mlf_status_string(mlf_status status);

#ifdef __cplusplus
}
#endif
#endif /* MLFABRIC_H */
