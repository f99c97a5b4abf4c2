// Dense hot path for gfx950: ordered K-way aggregate, ordered server apply, the
// fused aggregate + apply and the grouped apply of a whole scheduled batch, as
// one family of streaming kernels; optionally with the squared norms the
// scheduler needs reduced in the same pass, and the exact server-replica
// distance as a kernel of its own.
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

#include <atomic>

#include "mlfabric.h"

#pragma clang fp contract(off)

// Launch shapes: lanes per workgroup, groups per lane and tile, and number of
// updates whose loads are issued before any is consumed.  They are macros so that
// a sweep can rebuild the library with other values; the defaults are the best
// of such sweeps on MI355X (small workgroups, 32 loads in flight per lane).
#ifndef MLF_SHAPE_F32
#define MLF_SHAPE_F32 64, 2, 16
#endif
#ifndef MLF_SHAPE_BF16V4      // bfloat16, 4 elements per lane and group
#define MLF_SHAPE_BF16V4 64, 2, 8
#endif
#ifndef MLF_SHAPE_NORMS       // variants that also reduce norms (one wavefront per workgroup)
#define MLF_SHAPE_NORMS 64, 2, 8
#endif
#ifndef MLF_SHAPE_BF16V8      // bfloat16, 8 elements per lane and group
#define MLF_SHAPE_BF16V8 256, 1, 8
#endif
// 0: model / momentum use streaming (no-reuse) accesses only when they are too
// large to stay in the 256 MiB Infinity Cache between calls; 1: never; 4: always.
#ifndef MLF_STATE_POLICY
#define MLF_STATE_POLICY 0
#endif

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

static_assert(MLF_MAX_K <= 64, "group boundaries are one bit per sequence position");

enum Op { kAggregate = 0, kAggregateApply = 1, kApplyOrdered = 2, kApplyGrouped = 3 };

// Model + momentum up to this size are left to the caches between calls.
constexpr long long kInfinityCacheBytes = 256ll << 20;
// Workgroups that walk the element-wise region (they stride over it).
constexpr long long kMaxScalarGroups = 4096;

// Kernel argument block.  The host has already applied the scheduler's order:
// u[t] / wt[t] belong to the t-th committed update (wt = 1 without weights:
// multiplying by 1 is exact, so the unweighted sum needs no kernel of its own).
struct DenseArgs {
    const void *u[MLF_MAX_K];
    float wt[MLF_MAX_K];
    float *model;
    float *momentum;
    float *out;
    unsigned long long group_end;   // kApplyGrouped: bit t set = position t closes a group
    double *partials;       // norms variants: two partial sums per workgroup
    long long n;            // elements
    long long n_vec;        // leading elements on the 128-bit path (0 if unaligned)
    unsigned tiles_vec;     // workgroups [0, tiles_vec) each own one 128-bit tile
    int M;                  // committed updates
    float lr;
    float mu;
};

struct F32 {
    typedef float elem;
    static constexpr int kVec = 4;      // elements per 128-bit group
};
// bfloat16 updates come in two lane layouts.  8 elements per lane: one 128-bit
// load per update, but a wavefront's 128-bit model / momentum accesses then
// interleave two to a cache line, which only the cached state policy absorbs.
// 4 elements per lane: 64-bit update loads, contiguous 128-bit state accesses;
// the layout for streamed state.
struct BF16V8 {
    typedef uint16_t elem;
    static constexpr int kVec = 8;
};
struct BF16V4 {
    typedef uint16_t elem;
    static constexpr int kVec = 4;
};

__device__ __forceinline__ float from_bits(uint32_t b) { return __uint_as_float(b); }

// Load one group of W consecutive update elements, widened to binary32.  An
// update is read exactly once, so its loads carry the non-temporal hint and do
// not displace the model from the caches.  `e` is the group's first element.
template <typename IN, int W>
__device__ __forceinline__ void load_update(float (&x)[W], const void *base, long long e)
{
    if constexpr (W == 1) {
        if constexpr (sizeof(typename IN::elem) == 4) {
            x[0] = __builtin_nontemporal_load(static_cast<const float *>(base) + e);
        } else {
            uint16_t b = __builtin_nontemporal_load(static_cast<const uint16_t *>(base) + e);
            x[0] = from_bits(static_cast<uint32_t>(b) << 16);
        }
    } else if constexpr (sizeof(typename IN::elem) == 4) {
        static_assert(W == 4, "binary32 groups hold 4 elements");
        f32x4 v = __builtin_nontemporal_load(
            reinterpret_cast<const f32x4 *>(static_cast<const float *>(base) + e));
        x[0] = v.x; x[1] = v.y; x[2] = v.z; x[3] = v.w;
    } else if constexpr (W == 4) {
        u32x2 v = __builtin_nontemporal_load(
            reinterpret_cast<const u32x2 *>(static_cast<const uint16_t *>(base) + e));
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            x[2 * j] = from_bits(v[j] << 16);
            x[2 * j + 1] = from_bits(v[j] & 0xffff0000u);
        }
    } else {
        static_assert(W == 8, "bfloat16 groups hold 4 or 8 elements");
        u32x4 v = __builtin_nontemporal_load(
            reinterpret_cast<const u32x4 *>(static_cast<const uint16_t *>(base) + e));
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[2 * j] = from_bits(v[j] << 16);             // low half: even element
            x[2 * j + 1] = from_bits(v[j] & 0xffff0000u);   // high half: odd element
        }
    }
}

// Model / momentum accesses.  STREAM marks them non-temporal as well: used when
// the state is too large to stay cached until the next call.
template <int W, int STREAM>
__device__ __forceinline__ void load_state(float (&x)[W], const float *base, long long e)
{
    if constexpr (W == 1) {
        x[0] = base[e];
    } else {
#pragma unroll
        for (int j = 0; j < W / 4; ++j) {
            const f32x4 *p = reinterpret_cast<const f32x4 *>(base + e + 4 * j);
            f32x4 v;
            if constexpr ((STREAM & 1) != 0) {
                v = __builtin_nontemporal_load(p);
            } else {
                v = *p;
            }
            x[4 * j] = v.x; x[4 * j + 1] = v.y; x[4 * j + 2] = v.z; x[4 * j + 3] = v.w;
        }
    }
}

template <int W, int STREAM>
__device__ __forceinline__ void store_state(float *base, long long e, const float (&x)[W])
{
    if constexpr (W == 1) {
        base[e] = x[0];
    } else {
#pragma unroll
        for (int j = 0; j < W / 4; ++j) {
            f32x4 v = {x[4 * j], x[4 * j + 1], x[4 * j + 2], x[4 * j + 3]};
            f32x4 *p = reinterpret_cast<f32x4 *>(base + e + 4 * j);
            if constexpr ((STREAM & 2) != 0) {
                __builtin_nontemporal_store(v, p);
            } else {
                *p = v;
            }
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

// Work of one lane on one tile: VPT groups of W elements, THREADS groups apart,
// so that each load instruction of a wavefront covers one contiguous span.
//   e0       first element of the region the groups are counted in
//   g0       this lane's first group in that region
//   n_groups groups in the region
template <typename IN, int W, int OP, bool HAS_H, int STREAM, bool NORMS, int THREADS, int VPT,
          int CH, bool FULL>
struct Tile {
    const DenseArgs &a;
    long long e[VPT];       // first element of each group
    bool ok[VPT];
    float acc[VPT][W];      // running sum   (aggregate, aggregate+apply)
    float w[VPT][W];        // model         (apply variants)
    float h[VPT][W];        // history       (apply variants with momentum)
    float w_old[VPT][W];    // model before the call (norms variants)

    __device__ __forceinline__ Tile(const DenseArgs &args, long long e0, long long g0,
                                    long long n_groups)
        : a(args)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            long long g = g0 + static_cast<long long>(v) * THREADS;
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
            // Grouped apply: a position opens a group when its predecessor closed
            // one; uniform over the wavefront (scalar tests of the bit mask).
            const int t = t0 + c;
            const bool closes = OP == kApplyGrouped && ((a.group_end >> t) & 1ull) != 0;
            const bool opens = OP == kApplyGrouped && (t == 0 || ((a.group_end >> (t - 1)) & 1ull) != 0);
#pragma unroll
            for (int v = 0; v < VPT; ++v) {
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    if constexpr (OP == kApplyOrdered) {
                        server_step<HAS_H>(w[v][j], h[v][j], x[c][v][j], a.lr, a.mu);
                    } else if constexpr (OP == kApplyGrouped) {
                        const float term = wt * x[c][v][j];
                        acc[v][j] = opens ? term : acc[v][j] + term;
                        if (closes) server_step<HAS_H>(w[v][j], h[v][j], acc[v][j], a.lr, a.mu);
                    } else {
                        const float term = wt * x[c][v][j];
                        // The first term starts the sum; later ones are added.
                        acc[v][j] = first ? term : acc[v][j] + term;
                    }
                }
            }
        }
    }

    // Remainder of the sequence in halving pieces; positions stay in order.
    template <int C>
    __device__ __forceinline__ void remainder(int &t)
    {
        if constexpr (C >= 1) {
            if (a.M - t >= C) {
                chunk<C>(t);
                t += C;
            }
            remainder<C / 2>(t);
        }
    }

    // `sums` (norms variants): this lane's running squared norms in binary64,
    //   [0] aggregate: out^2          apply variants: history^2 after the call
    //   [1] apply variants: (model after - model before)^2
    // A binary32 square is exact in binary64, so only the additions round.
    __device__ __forceinline__ void run(double (&sums)[2])
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
                    load_state<W, STREAM>(w[v], a.model, e[v]);
                    if constexpr (HAS_H) load_state<W, STREAM>(h[v], a.momentum, e[v]);
                }
            }
            if constexpr (NORMS) {
#pragma unroll
                for (int j = 0; j < W; ++j) w_old[v][j] = w[v][j];
            }
        }

        int t = 0;
        for (; t + CH <= a.M; t += CH) chunk<CH>(t);
        remainder<CH / 2>(t);

#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            if (!ok[v]) continue;
            if constexpr (OP == kAggregate) {
                store_state<W, STREAM>(a.out, e[v], acc[v]);
            } else {
                if constexpr (OP == kAggregateApply) {
#pragma unroll
                    for (int j = 0; j < W; ++j) {
                        server_step<HAS_H>(w[v][j], h[v][j], acc[v][j], a.lr, a.mu);
                    }
                    if (a.out != nullptr) store_state<W, STREAM>(a.out, e[v], acc[v]);
                }
                store_state<W, STREAM>(a.model, e[v], w[v]);
                if constexpr (HAS_H) store_state<W, STREAM>(a.momentum, e[v], h[v]);
            }
            if constexpr (NORMS) {
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    if constexpr (OP == kAggregate) {
                        const double x = acc[v][j];
                        sums[0] += x * x;
                    } else {
                        const double hh = h[v][j];
                        const double dw = static_cast<double>(w[v][j]) - static_cast<double>(w_old[v][j]);
                        sums[0] += hh * hh;
                        sums[1] += dw * dw;
                    }
                }
            }
        }
    }
};

// Workgroups are handed to the 8 XCDs (each with its own L2) in turn.  With
// RUN > 0 every XCD takes runs of RUN consecutive tiles instead of every eighth
// tile, so that the lines an L2 writes back lie together; the last, incomplete
// block of 8 * RUN workgroups keeps the plain numbering, which keeps the map
// one to one.  Used where model and momentum go through the caches (+5 % there;
// no gain, or a loss, where they are streamed).
#ifndef MLF_XCD_RUN
#define MLF_XCD_RUN 512
#endif

template <unsigned RUN>
__device__ __forceinline__ long long xcd_tile(unsigned block, unsigned tiles)
{
    if constexpr (RUN == 0) {
        return block;
    } else {
        constexpr unsigned kBlock = 8 * RUN;
        const unsigned first = block / kBlock * kBlock;
        if (first + kBlock > tiles) return block;
        const unsigned r = block - first;
        return first + (r % 8) * RUN + r / 8;
    }
}

// Workgroups [0, tiles_vec) take one tile each of the 128-bit region
// [0, n_vec); the remaining workgroups stride over the element-wise region
// [n_vec, n): the ragged tail, or everything when a pointer of the call is not
// 16-byte aligned.  Norms variants (one wavefront per workgroup) end with a
// shuffle reduction in a fixed order and one pair of partial sums per workgroup.
template <typename IN, int OP, bool HAS_H, int STREAM, bool NORMS, int THREADS, int VPT, int CH>
__global__ __launch_bounds__(THREADS) void dense_kernel(const DenseArgs a)
{
    static_assert(!NORMS || THREADS == 64, "norms are reduced within one wavefront");
    constexpr int WV = IN::kVec;
    constexpr long long kTile = static_cast<long long>(THREADS) * VPT;
    double sums[2] = {0.0, 0.0};
    if (blockIdx.x < a.tiles_vec) {
        const long long groups = a.n_vec / WV;
        constexpr unsigned kRun = (STREAM == 0 && OP != kAggregate) ? MLF_XCD_RUN : 0;
        const long long base = xcd_tile<kRun>(blockIdx.x, a.tiles_vec) * kTile;
        if (base + kTile <= groups) {
            Tile<IN, WV, OP, HAS_H, STREAM, NORMS, THREADS, VPT, CH, true>(a, 0, base + threadIdx.x, groups).run(sums);
        } else {
            Tile<IN, WV, OP, HAS_H, STREAM, NORMS, THREADS, VPT, CH, false>(a, 0, base + threadIdx.x, groups).run(sums);
        }
    } else {
        const long long groups = a.n - a.n_vec;
        const long long stride = static_cast<long long>(gridDim.x - a.tiles_vec) * kTile;
        for (long long base = (blockIdx.x - a.tiles_vec) * kTile; base < groups; base += stride) {
            Tile<IN, 1, OP, HAS_H, STREAM, NORMS, THREADS, VPT, CH, false>(a, a.n_vec, base + threadIdx.x, groups).run(sums);
        }
    }
    if constexpr (NORMS) {
        double s0 = sums[0], s1 = sums[1];
        for (int off = 32; off > 0; off >>= 1) {
            s0 += __shfl_down(s0, off, 64);
            s1 += __shfl_down(s1, off, 64);
        }
        if (threadIdx.x == 0) {
            a.partials[2 * static_cast<size_t>(blockIdx.x)] = s0;
            a.partials[2 * static_cast<size_t>(blockIdx.x) + 1] = s1;
        }
    }
}

// Sums pairs of partial sums in a fixed order, so that the norms of a call are
// reproducible bit for bit for a given launch shape.  Workgroup b takes the
// pairs [b * slice, (b + 1) * slice) (cut at n_partials): lane i adds the
// pairs i, i + 1024, ... of the slice in turn, then a tree over the lanes; the
// result goes to out[2b] (and out[2b + 1] if n_out > 1).  A long list is
// reduced in two launches: kFinishSlices slices, then their sums.
constexpr int kFinishThreads = 1024;
constexpr unsigned kFinishSlices = 64;
constexpr unsigned kFinishTwoStageMin = 16384;   // pairs; below this one workgroup does it all

__global__ __launch_bounds__(kFinishThreads) void norms_finish_kernel(const double *partials,
                                                                      unsigned n_partials,
                                                                      unsigned slice, double *out,
                                                                      int n_out)
{
    __shared__ double tree[2][kFinishThreads];
    typedef double f64x2 __attribute__((ext_vector_type(2)));
    const f64x2 *pairs = reinterpret_cast<const f64x2 *>(partials);
    const unsigned begin = min(blockIdx.x * slice, n_partials);
    const unsigned end = min(begin + slice, n_partials);
    double s0 = 0.0, s1 = 0.0;
    // Eight loads in flight per lane; the additions keep their order.
    for (unsigned j0 = begin + threadIdx.x; j0 < end; j0 += kFinishThreads * 8) {
        f64x2 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned j = j0 + u * kFinishThreads;
            v[u] = j < end ? pairs[j] : f64x2{0.0, 0.0};
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            s0 += v[u].x;
            s1 += v[u].y;
        }
    }
    tree[0][threadIdx.x] = s0;
    tree[1][threadIdx.x] = s1;
    __syncthreads();
    for (int half = kFinishThreads / 2; half > 0; half >>= 1) {
        if (threadIdx.x < static_cast<unsigned>(half)) {
            tree[0][threadIdx.x] += tree[0][threadIdx.x + half];
            tree[1][threadIdx.x] += tree[1][threadIdx.x + half];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out[2 * static_cast<size_t>(blockIdx.x)] = tree[0][0];
        if (n_out > 1) out[2 * static_cast<size_t>(blockIdx.x) + 1] = tree[1][0];
    }
}

// Launches the reduction of `n_partials` pairs at `partials` into out[0..n_out).
// The kFinishSlices pairs after the capacity of the list are the scratch of the
// two-stage form.
bool finish_norms(double *partials, unsigned n_partials, size_t capacity, double *out, int n_out,
                  hipStream_t stream)
{
    if (n_partials >= kFinishTwoStageMin) {
        double *slices = partials + 2 * capacity;
        const unsigned slice = (n_partials + kFinishSlices - 1) / kFinishSlices;
        norms_finish_kernel<<<dim3(kFinishSlices), dim3(kFinishThreads), 0, stream>>>(
            partials, n_partials, slice, slices, 2);
        if (hipGetLastError() != hipSuccess) return false;
        norms_finish_kernel<<<dim3(1), dim3(kFinishThreads), 0, stream>>>(
            slices, kFinishSlices, kFinishSlices, out, n_out);
    } else {
        norms_finish_kernel<<<dim3(1), dim3(kFinishThreads), 0, stream>>>(
            partials, n_partials, n_partials, out, n_out);
    }
    return hipGetLastError() == hipSuccess;
}

// Exact server-replica divergence (Sec. 3.3 / 5.3: bounded consistency keeps
// ||w_s - w_r||_2 below Div_max): squared distance of two binary32 vectors.
// Same reduction scheme as the norms variants: one wavefront per workgroup, a
// pair of partial sums per workgroup (the second stays 0), fixed order.
constexpr int kDivUnroll = 4;       // 128-bit groups per lane and vector

__global__ __launch_bounds__(64) void divergence_kernel(const float *__restrict__ x,
                                                        const float *__restrict__ y, long long n,
                                                        long long n_vec, unsigned tiles_vec,
                                                        double *partials)
{
    double sum = 0.0;
    if (blockIdx.x < tiles_vec) {
        const long long groups = n_vec / 4;
        const long long base = static_cast<long long>(blockIdx.x) * 64 * kDivUnroll + threadIdx.x;
        f32x4 a[kDivUnroll], b[kDivUnroll];
#pragma unroll
        for (int u = 0; u < kDivUnroll; ++u) {
            const long long g = base + u * 64;
            const bool ok = g < groups;
            a[u] = ok ? __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(x) + g) : f32x4{0, 0, 0, 0};
            b[u] = ok ? __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(y) + g) : f32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kDivUnroll; ++u) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const double d = static_cast<double>(a[u][j]) - static_cast<double>(b[u][j]);
                sum += d * d;
            }
        }
    } else {
        const long long left = n - n_vec;
        const long long stride = static_cast<long long>(gridDim.x - tiles_vec) * 64;
        for (long long i = static_cast<long long>(blockIdx.x - tiles_vec) * 64 + threadIdx.x; i < left;
             i += stride) {
            const double d = static_cast<double>(x[n_vec + i]) - static_cast<double>(y[n_vec + i]);
            sum += d * d;
        }
    }
    for (int off = 32; off > 0; off >>= 1) sum += __shfl_down(sum, off, 64);
    if (threadIdx.x == 0) {
        partials[2 * static_cast<size_t>(blockIdx.x)] = sum;
        partials[2 * static_cast<size_t>(blockIdx.x) + 1] = 0.0;
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

// Workgroups a launch of this shape uses (tiles of the 128-bit region plus the
// workgroups of the element-wise region).
template <typename IN, int THREADS, int VPT>
void count_workgroups(const DenseArgs &a, long long &n_vec, long long &tiles_v, long long &tiles_s)
{
    constexpr long long kTile = static_cast<long long>(THREADS) * VPT;
    n_vec = a.n_vec / IN::kVec * IN::kVec;       // whole groups only
    tiles_v = (n_vec / IN::kVec + kTile - 1) / kTile;
    tiles_s = (a.n - n_vec + kTile - 1) / kTile;
    if (tiles_s > kMaxScalarGroups) tiles_s = kMaxScalarGroups;
}

template <typename IN, int OP, bool HAS_H, int STREAM, bool NORMS, int THREADS, int VPT, int CH>
mlf_status launch_shape(DenseArgs &a, hipStream_t stream, double *norms_out,
                        size_t partials_capacity)
{
    long long n_vec, tiles_v, tiles_s;
    count_workgroups<IN, THREADS, VPT>(a, n_vec, tiles_v, tiles_s);
    if (tiles_v + tiles_s > 0x7fffffffll) return MLF_EUNSUPPORTED;
    if (NORMS && static_cast<size_t>(tiles_v + tiles_s) > partials_capacity) return MLF_EINVAL;
    a.n_vec = n_vec;
    a.tiles_vec = static_cast<unsigned>(tiles_v);
    const unsigned grid = static_cast<unsigned>(tiles_v + tiles_s);
    if (grid > 0) {
        dense_kernel<IN, OP, HAS_H, STREAM, NORMS, THREADS, VPT, CH>
            <<<dim3(grid), dim3(THREADS), 0, stream>>>(a);
        if (hipGetLastError() != hipSuccess) return MLF_EHIP;
    }
    if constexpr (NORMS) {
        if (!finish_norms(a.partials, grid, partials_capacity, norms_out, OP == kAggregate ? 1 : 2, stream)) {
            return MLF_EHIP;
        }
    }
    return MLF_OK;
}

template <typename IN, int OP, bool HAS_H, int STREAM, bool NORMS>
mlf_status launch(DenseArgs &a, hipStream_t stream, double *norms_out, size_t partials_capacity)
{
    if constexpr (NORMS) {
        return launch_shape<IN, OP, HAS_H, STREAM, true, MLF_SHAPE_NORMS>(a, stream, norms_out,
                                                                          partials_capacity);
    } else if constexpr (sizeof(typename IN::elem) == 4) {
        return launch_shape<IN, OP, HAS_H, STREAM, false, MLF_SHAPE_F32>(a, stream, nullptr, 0);
    } else if constexpr (IN::kVec == 4) {
        return launch_shape<IN, OP, HAS_H, STREAM, false, MLF_SHAPE_BF16V4>(a, stream, nullptr, 0);
    } else {
        return launch_shape<IN, OP, HAS_H, STREAM, false, MLF_SHAPE_BF16V8>(a, stream, nullptr, 0);
    }
}

template <typename IN, int OP, int STREAM, bool NORMS>
mlf_status dispatch_state(DenseArgs &a, hipStream_t stream, double *norms_out, size_t capacity)
{
    if constexpr (OP == kAggregate) {
        return launch<IN, OP, false, STREAM, NORMS>(a, stream, norms_out, capacity);
    } else {
        return a.momentum != nullptr
                   ? launch<IN, OP, true, STREAM, NORMS>(a, stream, norms_out, capacity)
                   : launch<IN, OP, false, STREAM, NORMS>(a, stream, norms_out, capacity);
    }
}

template <int OP, bool NORMS = false>
mlf_status dispatch(DenseArgs &a, mlf_dtype dtype, hipStream_t stream, double *norms_out = nullptr,
                    size_t capacity = 0)
{
    // State that is too large to survive in the Infinity Cache until the next
    // call is streamed through; smaller state is left cacheable.  The output of
    // a plain aggregate is never read back by this library: always streamed.
    long long footprint = 0;
    if (a.model != nullptr) footprint += 4 * a.n;
    if (a.momentum != nullptr) footprint += 4 * a.n;
    if (a.out != nullptr) footprint += 4 * a.n;
    constexpr int kS = MLF_STATE_POLICY >= 2 ? MLF_STATE_POLICY - 1 : 3;
    const bool streaming = MLF_STATE_POLICY >= 2 ||
                           (MLF_STATE_POLICY == 0 && (OP == kAggregate || footprint > kInfinityCacheBytes));
    if (dtype == MLF_F32) {
        return streaming ? dispatch_state<F32, OP, kS, NORMS>(a, stream, norms_out, capacity)
                         : dispatch_state<F32, OP, 0, NORMS>(a, stream, norms_out, capacity);
    }
    return streaming ? dispatch_state<BF16V4, OP, kS, NORMS>(a, stream, norms_out, capacity)
                     : dispatch_state<BF16V8, OP, 0, NORMS>(a, stream, norms_out, capacity);
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
    a.n = n;
    a.n_vec = aligned16 ? n : 0;     // rounded down to whole groups at launch
    a.M = n_order;
    return MLF_OK;
}

// The groups must tile the committed sequence: positive lengths that add up to
// n_order.  Marks the closing position of every group in a.group_end.
bool mark_groups(DenseArgs &a, const int32_t *group_len, int n_groups, int n_order)
{
    long long covered = 0;
    a.group_end = 0;
    for (int j = 0; j < n_groups; ++j) {
        if (group_len[j] < 1 || covered + group_len[j] > n_order) return false;
        covered += group_len[j];
        a.group_end |= 1ull << (covered - 1);
    }
    return covered == n_order;
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
    a.group_end = 0;
    a.partials = nullptr;
    a.model = nullptr;
    a.momentum = nullptr;
    a.out = out;
    a.lr = 0.0f;
    a.mu = 0.0f;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dispatch<kAggregate>(a, dtype, s);
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
    a.group_end = 0;
    a.partials = nullptr;
    a.model = model;
    a.momentum = momentum;
    a.out = nullptr;
    a.lr = lr;
    a.mu = mu;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dispatch<kApplyOrdered>(a, dtype, s);
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
    a.group_end = 0;
    a.partials = nullptr;
    a.model = model;
    a.momentum = momentum;
    a.out = out_or_null;
    a.lr = lr;
    a.mu = mu;
    hipStream_t s = static_cast<hipStream_t>(stream);
    return dispatch<kAggregateApply>(a, dtype, s);
}

extern "C" mlf_status mlf_apply_grouped(float *model, float *momentum,
                                        const void *const *update_ptrs, int K, int64_t n,
                                        mlf_dtype dtype, const int32_t *order, int n_order,
                                        const float *weights, const int32_t *group_len,
                                        int n_groups, float lr, float mu, mlf_stream stream)
{
    if (model == nullptr || n_groups < 0 || (n_groups > 0 && group_len == nullptr)) return MLF_EINVAL;
    DenseArgs a;
    float *written[2] = {model, momentum};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, weights, written, 2);
    if (st != MLF_OK) return st;
    if (!mark_groups(a, group_len, n_groups, n_order)) return MLF_EINVAL;
    a.partials = nullptr;
    if (n == 0 || n_order == 0) return MLF_OK;
    a.model = model;
    a.momentum = momentum;
    a.out = nullptr;
    a.lr = lr;
    a.mu = mu;
    return dispatch<kApplyGrouped>(a, dtype, static_cast<hipStream_t>(stream));
}

// Partial sums a norms variant may need: one pair per workgroup of the
// (64 lanes x 2 groups) shape, for either layout of the elements.
static constexpr size_t norms_partials_capacity(long long n)
{
    return static_cast<size_t>(n / (64 * 2 * 4)) + 2 + static_cast<size_t>(kMaxScalarGroups);
}

extern "C" size_t mlf_norms_workspace_bytes(int64_t n)
{
    if (n < 0) return 0;
    return (norms_partials_capacity(n) + kFinishSlices) * 2 * sizeof(double);
}

extern "C" mlf_status mlf_aggregate_norm(const void *const *update_ptrs, int K, int64_t n,
                                         mlf_dtype dtype, const int32_t *order, int n_order,
                                         const float *weights, float *out, double *norm_sq,
                                         void *workspace, size_t workspace_bytes,
                                         mlf_stream stream)
{
    if (out == nullptr || norm_sq == nullptr) return MLF_EINVAL;
    if (n >= 0 && (workspace == nullptr || workspace_bytes < mlf_norms_workspace_bytes(n))) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(norm_sq) % 8 != 0) return MLF_EALIGN;
    DenseArgs a;
    float *written[1] = {out};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, weights, written, 1);
    if (st != MLF_OK) return st;
    a.group_end = 0;
    a.partials = static_cast<double *>(workspace);
    a.model = nullptr;
    a.momentum = nullptr;
    a.out = out;
    a.lr = 0.0f;
    a.mu = 0.0f;
    return dispatch<kAggregate, true>(a, dtype, static_cast<hipStream_t>(stream), norm_sq,
                                      norms_partials_capacity(n));
}

extern "C" mlf_status mlf_apply_grouped_norms(float *model, float *momentum,
                                              const void *const *update_ptrs, int K, int64_t n,
                                              mlf_dtype dtype, const int32_t *order, int n_order,
                                              const float *weights, const int32_t *group_len,
                                              int n_groups, float lr, float mu, double *norms_sq,
                                              void *workspace, size_t workspace_bytes,
                                              mlf_stream stream)
{
    if (model == nullptr || norms_sq == nullptr) return MLF_EINVAL;
    if (n_groups < 0 || (n_groups > 0 && group_len == nullptr)) return MLF_EINVAL;
    if (n >= 0 && (workspace == nullptr || workspace_bytes < mlf_norms_workspace_bytes(n))) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(norms_sq) % 8 != 0) return MLF_EALIGN;
    DenseArgs a;
    float *written[2] = {model, momentum};
    mlf_status st = prepare(a, update_ptrs, K, n, dtype, order, n_order, weights, written, 2);
    if (st != MLF_OK) return st;
    if (!mark_groups(a, group_len, n_groups, n_order)) return MLF_EINVAL;
    a.partials = static_cast<double *>(workspace);
    a.model = model;
    a.momentum = momentum;
    a.out = nullptr;
    a.lr = lr;
    a.mu = mu;
    return dispatch<kApplyGrouped, true>(a, dtype, static_cast<hipStream_t>(stream), norms_sq,
                                         norms_partials_capacity(n));
}

// Squared distance of two vectors with the partial sums in `partials` (room for
// norms_partials_capacity(n) + kFinishSlices pairs).  Every partial that is read
// has been written by this call, so the buffer needs no clearing.
static mlf_status divergence_launch(const float *w_server, const float *w_replica, long long n,
                                    double *dist_sq, double *partials, hipStream_t s)
{
    const bool aligned16 = reinterpret_cast<uintptr_t>(w_server) % 16 == 0 &&
                           reinterpret_cast<uintptr_t>(w_replica) % 16 == 0;
    const long long n_vec = aligned16 ? n / 4 * 4 : 0;
    const long long per_tile = 64 * kDivUnroll;                      // 128-bit groups per tile
    const long long tiles_v = (n_vec / 4 + per_tile - 1) / per_tile;
    long long tiles_s = (n - n_vec + 63) / 64;
    if (tiles_s > kMaxScalarGroups) tiles_s = kMaxScalarGroups;
    if (static_cast<size_t>(tiles_v + tiles_s) > norms_partials_capacity(n)) return MLF_EUNSUPPORTED;
    const unsigned grid = static_cast<unsigned>(tiles_v + tiles_s);
    if (grid > 0) {
        divergence_kernel<<<dim3(grid), dim3(64), 0, s>>>(w_server, w_replica, n, n_vec,
                                                         static_cast<unsigned>(tiles_v), partials);
        if (hipGetLastError() != hipSuccess) return MLF_EHIP;
    }
    return finish_norms(partials, grid, norms_partials_capacity(n), dist_sq, 1, s) ? MLF_OK : MLF_EHIP;
}

static mlf_status divergence_check(const float *w_server, const float *w_replica, long long n,
                                   const double *dist_sq)
{
    if (w_server == nullptr || w_replica == nullptr || dist_sq == nullptr || n < 0) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(w_server) % 4 != 0 || reinterpret_cast<uintptr_t>(w_replica) % 4 != 0 ||
        reinterpret_cast<uintptr_t>(dist_sq) % 8 != 0) {
        return MLF_EALIGN;
    }
    return MLF_OK;
}

extern "C" mlf_status mlf_divergence(const float *w_server, const float *w_replica, int64_t n,
                                     double *dist_sq, void *workspace, size_t workspace_bytes,
                                     mlf_stream stream)
{
    if (w_server == nullptr || w_replica == nullptr || dist_sq == nullptr || n < 0) return MLF_EINVAL;
    if (workspace == nullptr || workspace_bytes < mlf_norms_workspace_bytes(n)) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0) return MLF_EALIGN;
    const mlf_status st = divergence_check(w_server, w_replica, n, dist_sq);
    if (st != MLF_OK) return st;
    return divergence_launch(w_server, w_replica, n, dist_sq, static_cast<double *>(workspace),
                             static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------
// The divergence for callers that cannot allocate: its partial sums live in a
// file-scope device array instead of a caller's workspace.  Every GPU holds its
// own copy of the array at its own address; the address is looked up once per
// device (hipGetSymbolAddress, with that device current) and kept.  The array's
// name is only ever used in that lookup: host code passes the looked-up pointer.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes =
    (norms_partials_capacity(MLF_STATIC_MAX_N) + kFinishSlices) * 2 * sizeof(double);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<double *> g_scratch_ptr[kMaxDevices];

// The current device's copy of `scratch`.
static mlf_status static_scratch(double **out)
{
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess) return MLF_EHIP;
    if (device < 0 || device >= kMaxDevices) return MLF_EUNSUPPORTED;
    double *p = g_scratch_ptr[device].load(std::memory_order_acquire);
    if (p == nullptr) {
        void *address = nullptr;
        if (hipGetSymbolAddress(&address, HIP_SYMBOL(scratch)) != hipSuccess || address == nullptr) {
            return MLF_EHIP;
        }
        p = static_cast<double *>(address);
        // Threads that race here have looked up the same address.
        g_scratch_ptr[device].store(p, std::memory_order_release);
    }
    *out = p;
    return MLF_OK;
}

extern "C" mlf_status mlf_divergence_static(const float *w_server, const float *w_replica,
                                            int64_t n, double *dist_sq, mlf_stream stream)
{
    const mlf_status st = divergence_check(w_server, w_replica, n, dist_sq);
    if (st != MLF_OK) return st;
    if (n > MLF_STATIC_MAX_N) return MLF_EUNSUPPORTED;
    double *partials = nullptr;
    const mlf_status found = static_scratch(&partials);
    if (found != MLF_OK) return found;
    return divergence_launch(w_server, w_replica, n, dist_sq, partials,
                             static_cast<hipStream_t>(stream));
}

extern "C" const char *mlf_status_string(mlf_status status)
{
    switch (status) {
    case MLF_OK: return "MLF_OK";
    case MLF_EINVAL: return "MLF_EINVAL: invalid argument";
    case MLF_EALIGN: return "MLF_EALIGN: device pointer not aligned to its element size";
    case MLF_EUNSUPPORTED:
        return "MLF_EUNSUPPORTED: beyond a limit of the library (MLF_MAX_K updates or buffers, "
               "MLF_STATIC_MAX_N elements for the call without workspace)";
    case MLF_EHIP: return "MLF_EHIP: HIP launch failed";
    default: break;
    }
    return "unknown mlf_status";
}
