// Dense hot path for gfx950: ordered K-way aggregate, ordered server apply and
// the fused aggregate + apply, as one family of streaming kernels.
//
// Every element of the model is owned by exactly one lane, so the fixed
// per-element order of the sum (Sec. 5.2 of the paper: the scheduler's order is
// kept through aggregation) and of the server rule (Eq. 2, once per update) is
// a plain in-register loop; all parallelism is across elements.  Each update is
// read exactly once with 128-bit loads, model and momentum are read and written
// exactly once, whatever the number of updates: the kernels are bound by HBM
// bandwidth and by nothing else.
//
// Built with -ffp-contract=off: every product and every sum below is rounded
// on its own, as the definitions in mlfabric.h state.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "mlfabric.h"

#pragma clang fp contract(off)

// Launch shape (compile-time so that sweeps can rebuild with other values).
#ifndef MLF_VPT_F32      // 128-bit groups per lane and tile, binary32 updates
#define MLF_VPT_F32 2
#endif
#ifndef MLF_VPT_BF16     // 128-bit groups (8 elements) per lane and tile, bfloat16
#define MLF_VPT_BF16 1
#endif
#ifndef MLF_CHUNK        // updates whose loads are issued before any is consumed
#define MLF_CHUNK 8
#endif
#ifndef MLF_NT_LOAD      // updates are read once: bypass-friendly load hint
#define MLF_NT_LOAD 1
#endif
#ifndef MLF_NT_STORE
#define MLF_NT_STORE 0
#endif
#ifndef MLF_MAX_GRID     // workgroups per launch; tiles beyond it are strided
#define MLF_MAX_GRID (1 << 20)
#endif

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;

enum Op { kAggregate = 0, kAggregateApply = 1, kApplyOrdered = 2 };

// Kernel argument block.  The host has already applied the scheduler's order:
// u[t] / wt[t] belong to the t-th committed update.
struct DenseArgs {
    const void *u[MLF_MAX_K];
    float wt[MLF_MAX_K];
    float *model;
    float *momentum;
    float *out;
    long long n;            // elements
    long long n_vec;        // leading elements on the 128-bit path (0 if unaligned)
    int M;                  // committed updates
    float lr;
    float mu;
};

struct F32 {
    typedef float elem;
    static constexpr int kVec = 4;      // elements per 128-bit group
};
struct BF16 {
    typedef uint16_t elem;
    static constexpr int kVec = 8;
};

__device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }

template <typename T>
__device__ __forceinline__ T stream_load(const T *p)
{
#if MLF_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

template <typename T>
__device__ __forceinline__ void state_store(T *p, T v)
{
#if MLF_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Load one group of W consecutive update elements, widened to binary32.
// `e` is the index of the group's first element.
template <typename IN, int W>
__device__ __forceinline__ void load_update(float (&x)[W], const void *base, long long e)
{
    if constexpr (W == 1) {
        if constexpr (sizeof(typename IN::elem) == 4) {
            x[0] = stream_load(static_cast<const float *>(base) + e);
        } else {
            uint16_t b = stream_load(static_cast<const uint16_t *>(base) + e);
            x[0] = from_bits(static_cast<uint32_t>(b) << 16);
        }
    } else if constexpr (sizeof(typename IN::elem) == 4) {
        static_assert(W == 4, "binary32 groups hold 4 elements");
        f32x4 v = stream_load(reinterpret_cast<const f32x4 *>(static_cast<const float *>(base) + e));
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else {
        static_assert(W == 8, "bfloat16 groups hold 8 elements");
        u32x4 v = stream_load(reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(base) + e));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[2 * j] = from_bits(v[j] << 16);             // low half: even element
            x[2 * j + 1] = from_bits(v[j] & 0xffff0000u);   // high half: odd element
        }
    }
}

template <int W>
__device__ __forceinline__ void load_state(float (&x)[W], const float *base, long long e)
{
    if constexpr (W == 1) {
        x[0] = base[e];
    } else {
#pragma unroll
        for (int j = 0; j < W / 4; ++j) {
            f32x4 v = *reinterpret_cast<const f32x4 *>(base + e + 4 * j);
            x[4 * j] = v.x; x[4 * j + 1] = v.y; x[4 * j + 2] = v.z; x[4 * j + 3] = v.w;
        }
    }
}

template <int W>
__device__ __forceinline__ void store_state(float *base, long long e, const float (&x)[W])
{
    if constexpr (W == 1) {
        base[e] = x[0];
    } else {
#pragma unroll
        for (int j = 0; j < W / 4; ++j) {
            f32x4 v = {x[4 * j], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]};
            state_store(reinterpret_cast<f32x4 *>(base + e + 4 * j), v);
        }
    }
}

// One server step (Eq. 2 with u = -lr g): four separately rounded operations.
template <bool HAS_H>
__device__ __forceinline__ void server_step(float &w, float &h, float g, float lr, float mu)
{
    float q = lr * g;
    if constexpr (HAS_H) {
        float p = mu * h;
        h = p - q;
        w = w + h;
    } else {
        w = w - q;
    }
}

// Work of one lane on one tile: VPT groups of W elements, kThreads groups apart,
// so that each load instruction of a wavefront covers one contiguous span.
//   e0       first element of the region the groups are counted in
//   g0       this lane's first group in that region
//   n_groups groups in the region
template <typename IN, int W, int OP, bool WEIGHTED, bool HAS_H, int VPT, bool FULL>
struct Tile {
    const DenseArgs &a;
    long long e[VPT];       // first element of each group
    bool ok[VPT];
    float acc[VPT][W];      // running sum   (aggregate, aggregate+apply)
    float w[VPT][W];        // model         (apply variants)
    float h[VPT][W];        // history       (apply variants with momentum)

    __device__ __forceinline__ Tile(const DenseArgs &args, long long e0, long long g0,
                                    long long n_groups)
        : a(args)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            long long g = g0 + static_cast<long long>(v) * kThreads;
            ok[v] = FULL || g < n_groups;
            e[v] = e0 + g * W;
        }
    }

    // Consume C updates starting at position t0 of the sequence: all loads
    // first (memory-level parallelism), then the arithmetic in sequence order.
    template <int C>
    __device__ __forceinline__ void chunk(int t0)
    {
        float x[C][VPT][W];
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const void *p = a.u[t0 + c];
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
                if (ok[v]) {
                    load_update<IN, W>(x[c][v], p, e[v]);
                } else {
#pragma unroll
                    for (int j = 0; j < W; ++j) x[c][v][j] = 0.0f;
                }
            }
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float wt = a.wt[t0 + c];
            const bool first = (c == 0) && (t0 == 0);
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    if constexpr (OP == kApplyOrdered) {
                        server_step<HAS_H>(w[v][j], h[v][j], x[c][v][j], a.lr, a.mu);
                    } else {
                        float term = x[c][v][j];
                        if constexpr (WEIGHTED) term = wt * term;
                        // The first term starts the sum; later ones are added.
                        acc[v][j] = first ? term : acc[v][j] + term;
                    }
                }
            }
        }
    }

    __device__ __forceinline__ void run()
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
#pragma unroll
            for (int j = 0; j < W; ++j) {
                acc[v][j] = 0.0f;
                w[v][j] = 0.0f;
                h[v][j] = 0.0f;
            }
            if constexpr (OP != kAggregate) {
                if (ok[v]) {
                    load_state<W>(w[v], a.model, e[v]);
                    if constexpr (HAS_H) load_state<W>(h[v], a.momentum, e[v]);
                }
            }
        }

        int t = 0;
        for (; t + MLF_CHUNK <= a.M; t += MLF_CHUNK) chunk<MLF_CHUNK>(t);
        // Remainder in halving pieces; positions stay in sequence order.
        if constexpr (MLF_CHUNK > 16) { if (a.M - t >= 16) { chunk<16>(t); t += 16; } }
        if constexpr (MLF_CHUNK > 8) { if (a.M - t >= 8) { chunk<8>(t); t += 8; } }
        if constexpr (MLF_CHUNK > 4) { if (a.M - t >= 4) { chunk<4>(t); t += 4; } }
        if constexpr (MLF_CHUNK > 2) { if (a.M - t >= 2) { chunk<2>(t); t += 2; } }
        if constexpr (MLF_CHUNK > 1) { if (a.M - t >= 1) { chunk<1>(t); t += 1; } }

#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            if (!ok[v]) continue;
            if constexpr (OP == kAggregate) {
                store_state<W>(a.out, e[v], acc[v]);
            } else {
                if constexpr (OP == kAggregateApply) {
#pragma unroll
                    for (int j = 0; j < W; ++j) {
                        server_step<HAS_H>(w[v][j], h[v][j], acc[v][j], a.lr, a.mu);
                    }
                    if (a.out != nullptr) store_state<W>(a.out, e[v], acc[v]);
                }
                store_state<W>(a.model, e[v], w[v]);
                if constexpr (HAS_H) store_state<W>(a.momentum, e[v], h[v]);
            }
        }
    }
};

template <typename IN, int OP, bool WEIGHTED, bool HAS_H, int VPT>
__global__ __launch_bounds__(kThreads) void dense_kernel(const DenseArgs a)
{
    constexpr int WV = IN::kVec;
    constexpr long long kTile = static_cast<long long>(kThreads) * VPT;
    const long long stride = static_cast<long long>(gridDim.x) * kTile;

    // 128-bit region: elements [0, n_vec), in groups of WV.
    const long long groups_v = a.n_vec / WV;
    for (long long base = blockIdx.x * kTile; base < groups_v; base += stride) {
        if (base + kTile <= groups_v) {
            Tile<IN, WV, OP, WEIGHTED, HAS_H, VPT, true>(a, 0, base + threadIdx.x, groups_v).run();
        } else {
            Tile<IN, WV, OP, WEIGHTED, HAS_H, VPT, false>(a, 0, base + threadIdx.x, groups_v).run();
        }
    }
    // Element-wise region: [n_vec, n) -- the ragged tail, or everything when a
    // pointer of the call is not 16-byte aligned.
    const long long groups_s = a.n - a.n_vec;
    for (long long base = blockIdx.x * kTile; base < groups_s; base += stride) {
        Tile<IN, 1, OP, WEIGHTED, HAS_H, VPT, false>(a, a.n_vec, base + threadIdx.x, groups_s).run();
    }
}

// ---------------------------------------------------------------------------
// Host side: validation, order applied to the pointer / weight tables, launch.
// ---------------------------------------------------------------------------

struct Range {
    uintptr_t lo, hi;
};

bool overlap(Range a, Range b) { return a.lo < b.hi && b.lo < a.hi; }

Range range_of(const void *p, long long n, size_t elem)
{
    uintptr_t lo = reinterpret_cast<uintptr_t>(p);
    return Range{lo, lo + static_cast<uintptr_t>(n) * elem};
}

template <typename IN, int OP, bool WEIGHTED, bool HAS_H>
mlf_status launch(const DenseArgs &a, hipStream_t stream)
{
    constexpr int VPT = sizeof(typename IN::elem) == 4 ? MLF_VPT_F32 : MLF_VPT_BF16;
    constexpr long long kTile = static_cast<long long>(kThreads) * VPT;
    long long tiles_v = (a.n_vec / IN::kVec + kTile - 1) / kTile;
    long long tiles_s = (a.n - a.n_vec + kTile - 1) / kTile;
    long long grid = tiles_v > tiles_s ? tiles_v : tiles_s;
    if (grid < 1) grid = 1;
    if (grid > MLF_MAX_GRID) grid = MLF_MAX_GRID;
    dense_kernel<IN, OP, WEIGHTED, HAS_H, VPT>
        <<<dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, stream>>>(a);
    return hipGetLastError() == hipSuccess ? MLF_OK : MLF_EHIP;
}

template <typename IN, int OP>
mlf_status dispatch(const DenseArgs &a, bool weighted, hipStream_t stream)
{
    const bool has_h = a.momentum != nullptr;
    if constexpr (OP == kAggregate) {
        return weighted ? launch<IN, OP, true, false>(a, stream)
                        : launch<IN, OP, false, false>(a, stream);
    } else if constexpr (OP == kApplyOrdered) {
        return has_h ? launch<IN, OP, false, true>(a, stream)
                     : launch<IN, OP, false, false>(a, stream);
    } else {
        if (weighted) {
            return has_h ? launch<IN, OP, true, true>(a, stream)
                         : launch<IN, OP, true, false>(a, stream);
        }
        return has_h ? launch<IN, OP, false, true>(a, stream)
                     : launch<IN, OP, false, false>(a, stream);
    }
}

// Validates the arguments shared by the three dense calls and fills `a`.
// `written[]` are the binary32 vectors the call writes (NULL entries skipped).
mlf_status prepare(DenseArgs &a, const void *const *update_ptrs, int K, long long n,
                   mlf_dtype dtype, const int32_t *order, int n_order, const float *weights,
                   float *const *written, int n_written)
{
    if (K < 1 || n < 0 || n_order < 0 || n_order > K) return MLF_EINVAL;
    if (K > MLF_MAX_K) return MLF_EUNSUPPORTED;
    if (dtype != MLF_F32 && dtype != MLF_BF16) return MLF_EINVAL;
    if (update_ptrs == nullptr || (n_order > 0 && order == nullptr)) return MLF_EINVAL;
    const size_t esz = dtype == MLF_F32 ? 4 : 2;

    bool seen[MLF_MAX_K] = {false};
    bool aligned16 = true;
    for (int t = 0; t < n_order; ++t) {
        const int j = order[t];
        if (j < 0 || j >= K || seen[j]) return MLF_EINVAL;
        seen[j] = true;
        const void *p = update_ptrs[j];
        if (p == nullptr) return MLF_EINVAL;
        if (reinterpret_cast<uintptr_t>(p) % esz != 0) return MLF_EALIGN;
        aligned16 = aligned16 && reinterpret_cast<uintptr_t>(p) % 16 == 0;
        a.u[t] = p;
        a.wt[t] = weights != nullptr ? weights[j] : 1.0f;
    }
    for (int t = n_order; t < MLF_MAX_K; ++t) {
        a.u[t] = nullptr;
        a.wt[t] = 0.0f;
    }
    for (int i = 0; i < n_written; ++i) {
        if (written[i] == nullptr) continue;
        if (reinterpret_cast<uintptr_t>(written[i]) % 4 != 0) return MLF_EALIGN;
        aligned16 = aligned16 && reinterpret_cast<uintptr_t>(written[i]) % 16 == 0;
        const Range r = range_of(written[i], n, 4);
        for (int k = i + 1; k < n_written; ++k) {
            if (written[k] != nullptr && overlap(r, range_of(written[k], n, 4))) return MLF_EINVAL;
        }
        for (int t = 0; t < n_order; ++t) {
            if (overlap(r, range_of(a.u[t], n, esz))) return MLF_EINVAL;
        }
    }
    const int vec = dtype == MLF_F32 ? F32::kVec : BF16::kVec;
    a.n = n;
    a.n_vec = aligned16 ? (n / vec) * vec : 0;
    a.M = n_order;
    return MLF_OK;
}

}  // namespace

extern "C" mlf_status mlf_aggregate(const void *const *update_ptrs, int K, int64_t n,
                                    mlf_dtype dtype, const int32_t *order, int n_order,
                                    const float *weights, float *out, mlf_stream stream)
{
    if (out == nullptr) return MLF_EINVAL;
    DenseArgs a;
    float *written[1] = {out};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, weights, written, 1);
    if (st != MLF_OK) return st;
    if (n == 0) return MLF_OK;
    a.model = nullptr;
    a.momentum = nullptr;
    a.out = out;
    a.lr = 0.0f;
    a.mu = 0.0f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dtype == MLF_F32 ? dispatch<F32, kAggregate>(a, weights != nullptr, s)
                            : dispatch<BF16, kAggregate>(a, weights != nullptr, s);
}

extern "C" mlf_status mlf_apply_ordered(float *model, float *momentum,
                                        const void *const *update_ptrs, int K, int64_t n,
                                        mlf_dtype dtype, const int32_t *order, int n_order,
                                        float lr, float mu, mlf_stream stream)
{
    if (model == nullptr) return MLF_EINVAL;
    DenseArgs a;
    float *written[2] = {model, momentum};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, nullptr, written, 2);
    if (st != MLF_OK) return st;
    if (n == 0 || n_order == 0) return MLF_OK;
    a.model = model;
    a.momentum = momentum;
    a.out = nullptr;
    a.lr = lr;
    a.mu = mu;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dtype == MLF_F32 ? dispatch<F32, kApplyOrdered>(a, false, s)
                            : dispatch<BF16, kApplyOrdered>(a, false, s);
}

extern "C" mlf_status mlf_aggregate_apply(float *model, float *momentum, float *out_or_null,
                                          const void *const *update_ptrs, int K, int64_t n,
                                          mlf_dtype dtype, const int32_t *order, int n_order,
                                          const float *weights, float lr, float mu,
                                          mlf_stream stream)
{
    if (model == nullptr) return MLF_EINVAL;
    DenseArgs a;
    float *written[3] = {model, momentum, out_or_null};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, weights, written, 3);
    if (st != MLF_OK) return st;
    if (n == 0) return MLF_OK;
    a.model = model;
    a.momentum = momentum;
    a.out = out_or_null;
    a.lr = lr;
    a.mu = mu;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dtype == MLF_F32 ? dispatch<F32, kAggregateApply>(a, weights != nullptr, s)
                            : dispatch<BF16, kAggregateApply>(a, weights != nullptr, s);
}

extern "C" const char *mlf_status_string(mlf_status status)
{
    switch (status) {
    case MLF_OK: return "MLF_OK";
    case MLF_EINVAL: return "MLF_EINVAL: invalid argument";
    case MLF_EALIGN: return "MLF_EALIGN: device pointer not aligned to its element size";
    case MLF_EUNSUPPORTED: return "MLF_EUNSUPPORTED: more than MLF_MAX_K updates or buffers";
    case MLF_EHIP: return "MLF_EHIP: HIP launch failed";
    }
    return "unknown mlf_status";
}
