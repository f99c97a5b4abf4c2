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
// exactly once, whatever the number of updates: the kernels move exactly their
// algorithmic bytes and are bound by the memory system (hardware counters on 32
// updates of 61 M elements: vector units busy 16 to 27 % of the time, wavefronts
// waiting on memory for 50 to 80 % of theirs, every request a full line, no
// reuse in the L2).
//
// Built with -ffp-contract=off: every product and every sum below is rounded
// on its own, as the definitions in mlfabric.h state.
#include <hip/hip_runtime.h>

#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "launch.h"
#include "mlfabric.h"

#pragma clang fp contract(off)

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

static_assert(MLF_MAX_K <= 64, "group boundaries are one bit per sequence position");

enum Op { kAggregate = 0, kAggregateApply = 1, kApplyOrdered = 2, kApplyGrouped = 3 };
// Which squared norms a kernel reduces besides its pass: none; those of the call
// (one pair per workgroup); or those and one per committed update.
enum Norms { kNoNorms = 0, kCallNorms = 1, kUpdateNorms = 2 };

// Model + momentum up to this size are left to the caches between calls.
constexpr long long kInfinityCacheBytes = 256ll << 20;
// Workgroups that walk the element-wise region (they stride over it).
constexpr long long kMaxScalarGroups = 4096;
// Elements in the smallest tile of any launch shape (64 lanes x 1 group x 4).
constexpr long long kMinTileElements = 256;
// Update-norm variants: doubles in a workgroup's row of partial sums (the two
// sums of the call, then one per committed update), and the most workgroups
// that ever walk the 128-bit region (wavefronts resident on the device: a few
// per SIMD; the scratch is sized for this many rows plus the element-wise ones).
constexpr size_t kUpdateNormRow = 2 + MLF_MAX_K;
constexpr long long kUpdateNormMaxGroups = 8192;

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
    unsigned tiles_vec;     // tiles of the 128-bit region
    unsigned groups_vec;    // workgroups [0, groups_vec) take those tiles: one each (groups_vec ==
                            // tiles_vec), or in turn with stride groups_vec (update-norm variants)
    unsigned xcds;          // XCDs of the device (workgroups go to them in turn)
    int M;                  // committed updates
    float lr;
    float mu;
};

// The two tables of the argument block are indexed with run-time positions.
// They are read where the launch put them, in the kernel-argument segment
// (scalar loads, wavefront-uniform): the argument block is the kernel's only
// parameter and so starts that segment.  (Indexing the by-value parameter
// instead makes the compiler copy the whole block to per-lane scratch once the
// unrolled code refers to it often enough.)
#define MLF_KERNARG __attribute__((address_space(4)))
typedef const void *const MLF_KERNARG *UpdateTable;
typedef const float MLF_KERNARG *WeightTable;

__device__ __forceinline__ UpdateTable kernarg_updates()
{
    const char MLF_KERNARG *base = (const char MLF_KERNARG *)__builtin_amdgcn_kernarg_segment_ptr();
    return reinterpret_cast<UpdateTable>(base + offsetof(DenseArgs, u));
}

__device__ __forceinline__ WeightTable kernarg_weights()
{
    const char MLF_KERNARG *base = (const char MLF_KERNARG *)__builtin_amdgcn_kernarg_segment_ptr();
    return reinterpret_cast<WeightTable>(base + offsetof(DenseArgs, wt));
}

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

// Launch shapes.  A workgroup is one tile: THREADS lanes, each with VPT groups of
// consecutive elements, THREADS groups apart.  The committed sequence is consumed
// in blocks of HALF updates through two register buffers: the loads of the next
// block are issued before the current one is consumed.  A LIMITED shape is
// launched with a bounded number of workgroups per compute unit, by reserving
// that share of the unit's LDS for each (nothing is kept there); the number
// depends on the length of the sequence, see limited_per_cu().  The values are
// the best of sweeps on MI355X:
//
//  - binary32 updates, state streamed (more than the memory-side cache holds),
//    MANY updates committed (8 or more; 4 or more for the plain aggregate):
//    the narrowest tile (one 128-bit group per lane, 1 KiB per vector and
//    wavefront) and few one-wavefront workgroups per compute unit.  The fewer
//    and the narrower the tiles in flight, the shorter the stretch of every
//    vector that the chip works on at one time, and the cheaper the write-back
//    of model and momentum gets: an ordered apply of 32 updates of 61 M
//    elements runs at 0.773 of the peak with 4 per compute unit, 0.779 with 5,
//    0.765 with 6, 0.756 with 7 or more, and at 0.72 with 2 KiB tiles; the same
//    loads without the stores run at 0.89 either way.  With 4 (one per SIMD)
//    the end of a tile - the stores, and for the norms variants the binary64
//    squares, their reduction and the store of the pair - has nothing to hide
//    behind: the grouped apply with norms runs at 0.736 with 4 and 0.773 with
//    5.  Spreading the tiles in flight over 16 distant regions costs 6 %; tiles
//    of 512 bytes per vector lose 10-25 %;
//  - the same with FEW updates: the narrow tile then has too few loads in
//    flight whatever the number of workgroups, so the wide tile and the
//    unlimited occupancy are used (6.2-6.5 TB/s from 1 to 7 updates);
//  - bfloat16 updates, state streamed: a quarter of the traffic is stores and
//    64-bit update loads cover only 512 bytes per wavefront, so the wider tile
//    and the unlimited occupancy are kept (6.4 TB/s; the narrow shape at one
//    wavefront per SIMD drops to 3.4 TB/s);
//  - state that stays cached between calls: wider tiles, no limit.
//
// (The limit used to be set with the amdgpu_waves_per_eu attribute, one wavefront
// per SIMD.  Under that attribute the compiler produced wrong code for other
// instantiations of the tile template - a register that still held loaded data
// was reused as a temporary - so the dense kernels no longer use it.)
template <typename IN, bool STREAMED, int NORMS, bool MANY>
struct Shape;

template <int NORMS>
struct Shape<F32, true, NORMS, true> {      // streamed state, binary32, many updates
    static constexpr int kThreads = 64, kVpt = 1, kHalf = 8;
    static constexpr bool kLimited = true;
};
template <int NORMS>
struct Shape<F32, true, NORMS, false> {     // streamed state, binary32, few updates
    static constexpr int kThreads = 64, kVpt = 2, kHalf = 8;
    static constexpr bool kLimited = false;
};
template <int NORMS, bool MANY>
struct Shape<BF16V4, true, NORMS, MANY> {   // streamed state, bfloat16 updates
    static constexpr int kThreads = 64, kVpt = 2, kHalf = 4;
    static constexpr bool kLimited = false;
};
template <int NORMS, bool MANY>
struct Shape<F32, false, NORMS, MANY> {     // cached state, binary32 updates
    static constexpr int kThreads = 64, kVpt = 2, kHalf = 8;
    static constexpr bool kLimited = false;
};
template <int NORMS, bool MANY>
struct Shape<BF16V8, false, NORMS, MANY> {  // cached state, bfloat16 updates; with norms one wavefront per workgroup
    static constexpr int kThreads = NORMS != 0 ? 64 : 256, kVpt = NORMS != 0 ? 2 : 1, kHalf = 4;
    static constexpr bool kLimited = false;
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
template <typename IN, int W, int OP, bool HAS_H, int STREAM, int NORMS, int THREADS, int VPT,
          int HALF, bool FULL>
struct Tile {
    const DenseArgs &a;
    const UpdateTable u = kernarg_updates();    // a.u and a.wt, see UpdateTable
    const WeightTable wt_of = kernarg_weights();
    long long e[VPT];       // first element of each group
    bool ok[VPT];
    float acc[VPT][W];      // running sum   (aggregate, aggregate+apply)
    float w[VPT][W];        // model         (apply variants)
    float h[VPT][W];        // history       (apply variants with momentum)
    float w_old[VPT][W];    // model before the call (norms variants)
    double *update_sums;    // kUpdateNorms: LDS, [position][lane] running sum of squares of each update

    __device__ __forceinline__ Tile(const DenseArgs &args, long long e0, long long g0,
                                    long long n_groups, double *lds_update_sums = nullptr)
        : a(args), update_sums(lds_update_sums)
    {
#pragma unroll
        for (int v = 0; v < VPT; ++v) {
            long long g = g0 + static_cast<long long>(v) * THREADS;
            ok[v] = FULL || g < n_groups;
            e[v] = e0 + g * W;
        }
    }

    // Issues the loads of the C updates at positions t0 .. t0 + C - 1.
    template <int C>
    __device__ __forceinline__ void fetch(float (&x)[C][VPT][W], int t0)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const void *p = u[t0 + c];
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
    }

    // The arithmetic for the C updates at positions t0 .. t0 + C - 1, in
    // sequence order.
    template <int C>
    __device__ __forceinline__ void consume(const float (&x)[C][VPT][W], int t0)
    {
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const float wt = wt_of[t0 + c];
            const bool first = (c == 0) && (t0 == 0);
            // Grouped apply: a position opens a group when its predecessor closed
            // one; uniform over the wavefront (scalar tests of the bit mask).
            const int t = t0 + c;
            const bool closes = OP == kApplyGrouped && ((a.group_end >> t) & 1ull) != 0;
            const bool opens = OP == kApplyGrouped && (t == 0 || ((a.group_end >> (t - 1)) & 1ull) != 0);
            if constexpr (NORMS == kUpdateNorms) {
                // The update as it arrived (before its weight); a binary32 square
                // is exact in binary64.  Lanes without an element hold zeros.
                // (The fused multiply-add rounds once, as the separate addition
                // of the exact product would: the same bits, half the instructions.)
                double sq = 0.0;
#pragma unroll
                for (int v = 0; v < VPT; ++v) {
#pragma unroll
                    for (int j = 0; j < W; ++j) {
                        const double xx = x[c][v][j];
                        sq = __builtin_fma(xx, xx, sq);
                    }
                }
                // the lane's own slot: an LDS add that returns nothing, so nothing waits for it
                __hip_atomic_fetch_add(&update_sums[t * THREADS + threadIdx.x], sq, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
            }
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

    // What is left of the sequence after the whole blocks, in halving pieces
    // (loaded, then consumed); positions stay in order.
    template <int C>
    __device__ __forceinline__ void remainder(int &t)
    {
        if constexpr (C >= 1) {
            if (a.M - t >= C) {
                float x[C][VPT][W];
                fetch<C>(x, t);
                consume<C>(x, t);
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
            if constexpr (NORMS != kNoNorms) {
#pragma unroll
                for (int j = 0; j < W; ++j) w_old[v][j] = w[v][j];
            }
        }

        // Whole blocks of HALF updates alternate between two register buffers:
        // a block's loads are in flight while the block before it is consumed.
        const int M = a.M;
        int t = 0;
        if (M >= HALF) {
            float x0[HALF][VPT][W], x1[HALF][VPT][W];
            fetch<HALF>(x0, 0);
            for (;;) {
                if (t + 2 * HALF > M) {
                    consume<HALF>(x0, t);
                    t += HALF;
                    break;
                }
                fetch<HALF>(x1, t + HALF);
                consume<HALF>(x0, t);
                t += HALF;
                if (t + 2 * HALF > M) {
                    consume<HALF>(x1, t);
                    t += HALF;
                    break;
                }
                fetch<HALF>(x0, t + HALF);
                consume<HALF>(x1, t);
                t += HALF;
            }
        }
        remainder<HALF / 2>(t);

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
            if constexpr (NORMS != kNoNorms) {
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

// Workgroups are handed to the XCDs (each with its own L2) in turn.  With
// RUN > 0 every XCD takes runs of RUN consecutive tiles instead of every
// xcds-th tile, so that the lines an L2 writes back lie together; the last,
// incomplete block of xcds * RUN workgroups keeps the plain numbering, which
// keeps the map one to one.  Used where model and momentum go through the
// caches (+1 to 5 % there; no gain, or a loss, where they are streamed).
constexpr unsigned kXcdRun = 512;

template <unsigned RUN>
__device__ __forceinline__ long long xcd_tile(unsigned block, unsigned tiles, unsigned xcds)
{
    if constexpr (RUN == 0) {
        return block;
    } else {
        const unsigned per_block = xcds * RUN;
        const unsigned first = block / per_block * per_block;
        if (first + per_block > tiles) return block;
        const unsigned r = block - first;
        return first + (r % xcds) * RUN + r / xcds;
    }
}

// Workgroups [0, tiles_vec) take one tile each of the 128-bit region
// [0, n_vec); the remaining workgroups stride over the element-wise region
// [n_vec, n): the ragged tail, or everything when a pointer of the call is not
// 16-byte aligned.  Norms variants (one wavefront per workgroup) end with a
// shuffle reduction in a fixed order and one pair of partial sums per workgroup.
template <typename IN, int OP, bool HAS_H, int STREAM, int NORMS, int THREADS, int VPT, int HALF>
__device__ __forceinline__ void dense_body(const DenseArgs &a)
{
    static_assert(NORMS == kNoNorms || THREADS == 64, "norms are reduced within one wavefront");
    constexpr int WV = IN::kVec;
    constexpr long long kTile = static_cast<long long>(THREADS) * VPT;
    double sums[2] = {0.0, 0.0};
    // kUpdateNorms: one running sum per committed update and lane, in dynamic LDS.
    extern __shared__ double lds_update_sums[];
    double *update_sums = nullptr;
    if constexpr (NORMS == kUpdateNorms) {
        update_sums = lds_update_sums;
        for (int t = 0; t < a.M; ++t) update_sums[t * THREADS + threadIdx.x] = 0.0;
    }
    if (blockIdx.x < a.groups_vec) {
        const long long groups = a.n_vec / WV;
        constexpr unsigned kRun = (STREAM == 0 && OP != kAggregate && NORMS != kUpdateNorms) ? kXcdRun : 0;
        // (one tile per workgroup, except for the update-norm variants, whose
        // workgroups take the tiles in turn and keep their sums over all of them)
        for (unsigned tile = blockIdx.x; tile < a.tiles_vec; tile += a.groups_vec) {
            const long long base = xcd_tile<kRun>(tile, a.tiles_vec, a.xcds) * kTile;
            if (base + kTile <= groups) {
                Tile<IN, WV, OP, HAS_H, STREAM, NORMS, THREADS, VPT, HALF, true>(a, 0, base + threadIdx.x, groups, update_sums).run(sums);
            } else {
                Tile<IN, WV, OP, HAS_H, STREAM, NORMS, THREADS, VPT, HALF, false>(a, 0, base + threadIdx.x, groups, update_sums).run(sums);
            }
            if constexpr (NORMS != kUpdateNorms) break;
        }
    } else {
        const long long groups = a.n - a.n_vec;
        const long long stride = static_cast<long long>(gridDim.x - a.groups_vec) * kTile;
        for (long long base = (blockIdx.x - a.groups_vec) * kTile; base < groups; base += stride) {
            Tile<IN, 1, OP, HAS_H, STREAM, NORMS, THREADS, VPT, HALF, false>(a, a.n_vec, base + threadIdx.x, groups, update_sums).run(sums);
        }
    }
    if constexpr (NORMS != kNoNorms) {
        // One row of partial sums per workgroup: the two sums of the call, and
        // for the update-norm variants one per committed update after them.
        constexpr size_t kRow = NORMS == kUpdateNorms ? kUpdateNormRow : 2;
        double *row = a.partials + kRow * static_cast<size_t>(blockIdx.x);
        double s0 = sums[0], s1 = sums[1];
        for (int off = 32; off > 0; off >>= 1) {
            s0 += __shfl_down(s0, off, 64);
            s1 += __shfl_down(s1, off, 64);
        }
        if (threadIdx.x == 0) {
            row[0] = s0;
            row[1] = s1;
        }
        if constexpr (NORMS == kUpdateNorms) {
            for (int t = 0; t < a.M; ++t) {
                double u = update_sums[t * THREADS + threadIdx.x];
                for (int off = 32; off > 0; off >>= 1) u += __shfl_down(u, off, 64);
                if (threadIdx.x == 0) row[2 + t] = u;
            }
        }
    }
}

// The kernel proper.
template <typename IN, int OP, bool HAS_H, int STREAM, int NORMS, int THREADS, int VPT, int HALF>
__global__ __launch_bounds__(THREADS) void dense_kernel(const DenseArgs a)
{
    dense_body<IN, OP, HAS_H, STREAM, NORMS, THREADS, VPT, HALF>(a);
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
    const double *in = partials;
    if (n_partials >= kFinishTwoStageMin) {
        double *slices = partials + 2 * capacity;
        const unsigned slice = (n_partials + kFinishSlices - 1) / kFinishSlices;
        if (!launch_kernel(norms_finish_kernel, dim3(kFinishSlices), dim3(kFinishThreads), 0, stream, in,
                           n_partials, slice, slices, 2)) {
            return false;
        }
        in = slices;
        n_partials = kFinishSlices;
    }
    return launch_kernel(norms_finish_kernel, dim3(1), dim3(kFinishThreads), 0, stream, in, n_partials,
                         n_partials, out, n_out);
}

// The same for the rows of the update-norm variants: workgroup c sums column c
// of the `rows` rows (lane i adds rows i, i + 256, ... in turn, then a tree over
// the lanes).  Columns 0 and 1 are the sums of the call (column 1 is dropped when
// n_main == 1), column 2 + t belongs to the t-th committed update.
constexpr int kColumnThreads = 256;

__global__ __launch_bounds__(kColumnThreads) void update_norms_finish_kernel(const double *partials,
                                                                           unsigned rows,
                                                                           double *main_out, int n_main,
                                                                           double *update_out)
{
    __shared__ double tree[kColumnThreads];
    const unsigned c = blockIdx.x;
    double sum = 0.0;
    for (unsigned r0 = threadIdx.x; r0 < rows; r0 += kColumnThreads * 8) {
        double v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const unsigned r = r0 + u * kColumnThreads;
            v[u] = r < rows ? partials[kUpdateNormRow * static_cast<size_t>(r) + c] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) sum += v[u];
    }
    tree[threadIdx.x] = sum;
    __syncthreads();
    for (int half = kColumnThreads / 2; half > 0; half >>= 1) {
        if (threadIdx.x < static_cast<unsigned>(half)) tree[threadIdx.x] += tree[threadIdx.x + half];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        if (c >= 2) {
            update_out[c - 2] = tree[0];
        } else if (static_cast<int>(c) < n_main) {
            main_out[c] = tree[0];
        }
    }
}

// Exact server-replica divergence (Sec. 3.3 / 5.3: bounded consistency keeps
// ||w_s - w_r||_2 below Div_max): squared distance of two binary32 vectors.
// Same reduction scheme as the norms variants: one wavefront per workgroup, a
// pair of partial sums per workgroup (the second stays 0), fixed order.  The
// first `groups_vec` workgroups take the tiles of the 128-bit region in turn
// (tile, tile + groups_vec, ...): at most kDivMaxGroups of them, so that the
// partial sums stay few enough for ONE reduction launch behind the kernel (a
// second one costs 5 us, 6 % of this kernel on 61 M elements).
constexpr int kDivUnroll = 4;               // 128-bit groups per lane, vector and tile
constexpr long long kDivMaxGroups = 8192;   // workgroups of the 128-bit region

__global__ __launch_bounds__(64) void divergence_kernel(const float *__restrict__ x,
                                                        const float *__restrict__ y, long long n,
                                                        long long n_vec, unsigned tiles_vec,
                                                        unsigned groups_vec, double *partials)
{
    double sum = 0.0;
    if (blockIdx.x < groups_vec) {
        const long long groups = n_vec / 4;
        for (unsigned tile = blockIdx.x; tile < tiles_vec; tile += groups_vec) {
            const long long base = static_cast<long long>(tile) * 64 * kDivUnroll + threadIdx.x;
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
        }
    } else {
        const long long left = n - n_vec;
        const long long stride = static_cast<long long>(gridDim.x - groups_vec) * 64;
        for (long long i = static_cast<long long>(blockIdx.x - groups_vec) * 64 + threadIdx.x; i < left;
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

// XCDs of the current device (its workgroups are handed to them in turn);
// looked up once per device.  1 when the runtime cannot tell: tile numbering
// then stays plain.
unsigned xcd_count()
{
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cached[kMaxDevices];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return 1;
    int n = cached[device].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeNumberOfXccs, device) != hipSuccess || n < 1) n = 1;
        cached[device].store(n, std::memory_order_relaxed);
    }
    return static_cast<unsigned>(n);
}

// LDS of a compute unit of the current device, looked up once per device
// (gfx950: 160 KiB), and the unit it is handed out in (1,280 bytes there: a
// request is rounded up to it, measured through the occupancy it leaves).
constexpr size_t kLdsGranule = 1280;

size_t lds_per_cu()
{
    constexpr int kMaxDevices = 64;
    constexpr int kDefault = 160 * 1024;
    static std::atomic<int> cached[kMaxDevices];
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return kDefault;
    int n = cached[device].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, device) != hipSuccess ||
            n < 65536) {
            n = kDefault;
        }
        cached[device].store(n, std::memory_order_relaxed);
    }
    return static_cast<size_t>(n);
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

// Committed updates from which the streamed binary32 kernels use the narrow shape
// (MANY), and the workgroups per compute unit that shape is limited to.  Measured
// on 61 M elements (TB/s, wide shape | narrow shape limited to 4, 5, 6, 8, 12):
//   ordered apply  M = 6: 6.38 | 4.12 4.82 5.43 6.31 6.32     aggregate  M = 6: 6.36 | 4.01 4.68 5.27 5.79 6.74
//                  M = 8: 6.23 | 6.40 6.74 6.69 6.62 6.60                M = 8: 6.25 | 5.69 6.22 6.58 6.54 6.48
//                  M = 13: 6.18 | 5.58 6.20 6.58 6.63 6.62               M = 13: 6.09 | 5.06 5.69 6.20 6.71 6.48
//                  M = 16: 6.11 | 6.36 6.46 6.34 6.37 6.36               M = 16: 6.11 | 6.22 6.65 6.55 6.47 6.30
//                  M = 18: 6.04 | 5.93 6.36 6.44 6.36 6.36               M = 18: 6.03 | 5.84 6.39 6.61 6.43 6.30
//                  M = 32: 5.84 | 6.26 6.24 6.13 6.02 6.04               M = 32: 6.12 | 6.63 6.55 6.44 6.32 6.17
// The longer the sequence, the fewer workgroups should be in flight; a sequence
// that is a whole number of blocks wants fewer than its neighbours, whose
// remainder pieces are loaded only once the last whole block has been consumed.
//
// The update-norm variants walk the tiles with as many workgroups as are
// resident, and do best with the narrow shape from 16 updates on and one
// workgroup per SIMD (32 updates of 61 M elements: 0.70 of the peak with 4 per
// compute unit, 0.66 with 5, 0.65 with 6 or 8).
constexpr int kManyUpdates = 8, kManyUpdatesAggregate = 4, kManyUpdatesUpdateNorms = 16;

template <int NORMS>
inline unsigned limited_per_cu(int M)
{
    if (NORMS == kUpdateNorms) return 4;
    if (M < 8) return 12;               // (the plain aggregate only: as many as fit, about)
    if (M % 8 == 0 || M >= 24) return 5;
    return M >= 16 ? 6 : 8;
}

template <typename IN, int OP, bool HAS_H, int STREAM, int NORMS, bool MANY>
mlf_status launch_shape(DenseArgs &a, hipStream_t stream, double *norms_out, size_t partials_capacity,
                        double *update_norms_out)
{
    typedef Shape<IN, STREAM != 0, NORMS, MANY> S;
    static_assert(!S::kLimited || S::kThreads == 64, "the limit counts one-wavefront workgroups");
    static_assert(64 * S::kVpt * IN::kVec >= kMinTileElements || NORMS == kNoNorms, "a norms tile yields one partial pair");
    long long n_vec, tiles_v, tiles_s;
    count_workgroups<IN, S::kThreads, S::kVpt>(a, n_vec, tiles_v, tiles_s);
    if (tiles_v > 0xffffffffll) return MLF_EUNSUPPORTED;
    long long groups_v = tiles_v;
    // Dynamic LDS of a workgroup: the running sums of the update-norm variants,
    // and for a shape that limits the workgroups per compute unit at least that
    // share of the unit's LDS.
    size_t lds = 0;
    if constexpr (NORMS == kUpdateNorms) lds = static_cast<size_t>(a.M) * S::kThreads * sizeof(double);
    long long per_cu = 12;      // one-wavefront workgroups a compute unit holds when nothing limits them, about
    if constexpr (S::kLimited) {
        const size_t all = lds_per_cu();
        const size_t share = all / limited_per_cu<NORMS>(a.M) / kLdsGranule * kLdsGranule;
        if (lds < share) lds = share;
        per_cu = static_cast<long long>(all / ((lds + kLdsGranule - 1) / kLdsGranule * kLdsGranule));
    }
    if constexpr (NORMS == kUpdateNorms) {
        // As many workgroups (of one wavefront) as the device keeps resident.
        const long long resident = static_cast<long long>(cu_count()) * per_cu;
        const long long cap = resident < 1 ? 1024 : resident > kUpdateNormMaxGroups ? kUpdateNormMaxGroups : resident;
        if (groups_v > cap) groups_v = cap;
    }
    if (groups_v + tiles_s > 0x7fffffffll) return MLF_EUNSUPPORTED;
    if (NORMS != kNoNorms && static_cast<size_t>(groups_v + tiles_s) > partials_capacity) return MLF_EINVAL;
    a.n_vec = n_vec;
    a.tiles_vec = static_cast<unsigned>(tiles_v);
    a.groups_vec = static_cast<unsigned>(groups_v);
    a.xcds = xcd_count();
    const unsigned grid = static_cast<unsigned>(groups_v + tiles_s);
    if (grid > 0) {
        const bool ok = launch_kernel(dense_kernel<IN, OP, HAS_H, STREAM, NORMS, S::kThreads, S::kVpt, S::kHalf>,
                                      dim3(grid), dim3(S::kThreads), lds, stream, a);
        if (!ok) return MLF_EHIP;
    }
    if constexpr (NORMS == kCallNorms) {
        if (!finish_norms(a.partials, grid, partials_capacity, norms_out, OP == kAggregate ? 1 : 2, stream)) {
            return MLF_EHIP;
        }
    }
    if constexpr (NORMS == kUpdateNorms) {
        // (with no workgroup at all, n == 0, every sum is 0: rows = 0)
        if (!launch_kernel(update_norms_finish_kernel, dim3(2 + static_cast<unsigned>(a.M)), dim3(kColumnThreads), 0,
                           stream, a.partials, grid, norms_out, OP == kAggregate ? 1 : 2, update_norms_out)) {
            return MLF_EHIP;
        }
    }
    return MLF_OK;
}

template <typename IN, int OP, bool HAS_H, int STREAM, int NORMS>
mlf_status launch(DenseArgs &a, hipStream_t stream, double *norms_out, size_t partials_capacity,
                  double *update_norms_out)
{
    if constexpr (sizeof(typename IN::elem) == 4 && STREAM != 0) {
        if (a.M >= (NORMS == kUpdateNorms ? kManyUpdatesUpdateNorms : OP == kAggregate ? kManyUpdatesAggregate : kManyUpdates)) {
            return launch_shape<IN, OP, HAS_H, STREAM, NORMS, true>(a, stream, norms_out, partials_capacity,
                                                                    update_norms_out);
        }
    }
    return launch_shape<IN, OP, HAS_H, STREAM, NORMS, false>(a, stream, norms_out, partials_capacity,
                                                             update_norms_out);
}

template <typename IN, int OP, int STREAM, int NORMS>
mlf_status dispatch_state(DenseArgs &a, hipStream_t stream, double *norms_out, size_t capacity,
                          double *update_norms_out)
{
    if constexpr (OP == kAggregate) {
        return launch<IN, OP, false, STREAM, NORMS>(a, stream, norms_out, capacity, update_norms_out);
    } else {
        return a.momentum != nullptr
                   ? launch<IN, OP, true, STREAM, NORMS>(a, stream, norms_out, capacity, update_norms_out)
                   : launch<IN, OP, false, STREAM, NORMS>(a, stream, norms_out, capacity, update_norms_out);
    }
}

template <int OP, int NORMS = kNoNorms>
mlf_status dispatch(DenseArgs &a, mlf_dtype dtype, hipStream_t stream, double *norms_out = nullptr,
                    size_t capacity = 0, double *update_norms_out = nullptr)
{
    // State that is too large to survive in the memory-side cache until the
    // next call is streamed through (no-reuse hint on its loads and stores);
    // smaller state is left cacheable.  The output of a plain aggregate is
    // never read back by this library: always streamed.
    long long footprint = 0;
    if (a.model != nullptr) footprint += 4 * a.n;
    if (a.momentum != nullptr) footprint += 4 * a.n;
    if (a.out != nullptr) footprint += 4 * a.n;
    const bool streaming = OP == kAggregate || footprint > kInfinityCacheBytes;
    if (dtype == MLF_F32) {
        return streaming ? dispatch_state<F32, OP, 3, NORMS>(a, stream, norms_out, capacity, update_norms_out)
                         : dispatch_state<F32, OP, 0, NORMS>(a, stream, norms_out, capacity, update_norms_out);
    }
    return streaming ? dispatch_state<BF16V4, OP, 3, NORMS>(a, stream, norms_out, capacity, update_norms_out)
                     : dispatch_state<BF16V8, OP, 0, NORMS>(a, stream, norms_out, capacity, update_norms_out);
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

// Partial sums a norms variant may need: one pair per workgroup, and the
// smallest tile of any shape holds kMinTileElements elements.
static constexpr size_t norms_partials_capacity(long long n)
{
    return static_cast<size_t>(n / kMinTileElements) + 2 + static_cast<size_t>(kMaxScalarGroups);
}

// The same for the divergence kernel alone: its workgroups of the 128-bit
// region are capped whatever n is.
static constexpr size_t divergence_partials_capacity()
{
    return static_cast<size_t>(kDivMaxGroups) + static_cast<size_t>(kMaxScalarGroups);
}

extern "C" size_t mlf_norms_workspace_bytes(int64_t n)
{
    if (n < 0) return 0;
    return (norms_partials_capacity(n) + kFinishSlices) * 2 * sizeof(double);
}

// Rows of partial sums an update-norm variant may need, whatever the device.
static constexpr size_t update_norms_rows() { return static_cast<size_t>(kUpdateNormMaxGroups + kMaxScalarGroups); }

extern "C" size_t mlf_update_norms_workspace_bytes(int64_t n)
{
    if (n < 0) return 0;
    return update_norms_rows() * kUpdateNormRow * sizeof(double);
}

// mlf_aggregate_norm and mlf_aggregate_update_norms (update_norm_sq != NULL).
static mlf_status aggregate_with_norms(const void *const *update_ptrs, int K, int64_t n, mlf_dtype dtype,
                                       const int32_t *order, int n_order, const float *weights,
                                       float *out, double *norm_sq, double *update_norm_sq,
                                       bool per_update, void *workspace, size_t workspace_bytes,
                                       mlf_stream stream)
{
    if (out == nullptr || norm_sq == nullptr || (per_update && update_norm_sq == nullptr)) return MLF_EINVAL;
    const size_t need = per_update ? mlf_update_norms_workspace_bytes(n) : mlf_norms_workspace_bytes(n);
    if (n >= 0 && (workspace == nullptr || workspace_bytes < need)) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(norm_sq) % 8 != 0 ||
        reinterpret_cast<uintptr_t>(update_norm_sq) % 8 != 0) {
        return MLF_EALIGN;
    }
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    return per_update ? dispatch<kAggregate, kUpdateNorms>(a, dtype, s, norm_sq, update_norms_rows(), update_norm_sq)
                      : dispatch<kAggregate, kCallNorms>(a, dtype, s, norm_sq, norms_partials_capacity(n));
}

extern "C" mlf_status mlf_aggregate_norm(const void *const *update_ptrs, int K, int64_t n,
                                         mlf_dtype dtype, const int32_t *order, int n_order,
                                         const float *weights, float *out, double *norm_sq,
                                         void *workspace, size_t workspace_bytes,
                                         mlf_stream stream)
{
    return aggregate_with_norms(update_ptrs, K, n, dtype, order, n_order, weights, out, norm_sq, nullptr,
                                false, workspace, workspace_bytes, stream);
}

extern "C" mlf_status mlf_aggregate_update_norms(const void *const *update_ptrs, int K, int64_t n,
                                                 mlf_dtype dtype, const int32_t *order, int n_order,
                                                 const float *weights, float *out, double *norm_sq,
                                                 double *update_norm_sq, void *workspace,
                                                 size_t workspace_bytes, mlf_stream stream)
{
    return aggregate_with_norms(update_ptrs, K, n, dtype, order, n_order, weights, out, norm_sq,
                                update_norm_sq, true, workspace, workspace_bytes, stream);
}

// mlf_apply_grouped_norms and mlf_apply_grouped_update_norms.
static mlf_status apply_grouped_with_norms(float *model, float *momentum, const void *const *update_ptrs,
                                           int K, int64_t n, mlf_dtype dtype, const int32_t *order,
                                           int n_order, const float *weights, const int32_t *group_len,
                                           int n_groups, float lr, float mu, double *norms_sq,
                                           double *update_norm_sq, bool per_update, void *workspace,
                                           size_t workspace_bytes, mlf_stream stream)
{
    if (model == nullptr || norms_sq == nullptr || (per_update && update_norm_sq == nullptr)) return MLF_EINVAL;
    if (n_groups < 0 || (n_groups > 0 && group_len == nullptr)) return MLF_EINVAL;
    const size_t need = per_update ? mlf_update_norms_workspace_bytes(n) : mlf_norms_workspace_bytes(n);
    if (n >= 0 && (workspace == nullptr || workspace_bytes < need)) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace) % 16 != 0 || reinterpret_cast<uintptr_t>(norms_sq) % 8 != 0 ||
        reinterpret_cast<uintptr_t>(update_norm_sq) % 8 != 0) {
        return MLF_EALIGN;
    }
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    return per_update ? dispatch<kApplyGrouped, kUpdateNorms>(a, dtype, s, norms_sq, update_norms_rows(), update_norm_sq)
                      : dispatch<kApplyGrouped, kCallNorms>(a, dtype, s, norms_sq, norms_partials_capacity(n));
}

extern "C" mlf_status mlf_apply_grouped_norms(float *model, float *momentum,
                                              const void *const *update_ptrs, int K, int64_t n,
                                              mlf_dtype dtype, const int32_t *order, int n_order,
                                              const float *weights, const int32_t *group_len,
                                              int n_groups, float lr, float mu, double *norms_sq,
                                              void *workspace, size_t workspace_bytes,
                                              mlf_stream stream)
{
    return apply_grouped_with_norms(model, momentum, update_ptrs, K, n, dtype, order, n_order, weights,
                                    group_len, n_groups, lr, mu, norms_sq, nullptr, false, workspace,
                                    workspace_bytes, stream);
}

extern "C" mlf_status mlf_apply_grouped_update_norms(float *model, float *momentum,
                                                     const void *const *update_ptrs, int K, int64_t n,
                                                     mlf_dtype dtype, const int32_t *order, int n_order,
                                                     const float *weights, const int32_t *group_len,
                                                     int n_groups, float lr, float mu, double *norms_sq,
                                                     double *update_norm_sq, void *workspace,
                                                     size_t workspace_bytes, mlf_stream stream)
{
    return apply_grouped_with_norms(model, momentum, update_ptrs, K, n, dtype, order, n_order, weights,
                                    group_len, n_groups, lr, mu, norms_sq, update_norm_sq, true, workspace,
                                    workspace_bytes, stream);
}

// The scheduler's upper bound of the divergence a batch causes (Sec. 5.3),
// from the norms the calls above return: Eq. 2 unrolled over the batch's server
// steps gives w_after - w_before = (mu + ... + mu^S) h0 + sum_j c_j u_j with
// c_j = 1 + mu + ... + mu^(S-j), and u_j = -lr * (sum over group j of wt * g);
// the triangle inequality bounds the norm of the whole and of every u_j.  Host
// arithmetic only.
extern "C" mlf_status mlf_divergence_bound(double h_norm_sq, const double *update_norm_sq,
                                           const int32_t *order, int n_order, int K,
                                           const float *weights, const int32_t *group_len,
                                           int n_groups, float lr, float mu, double *bound)
{
    if (bound == nullptr || K < 1 || n_order < 0 || n_order > K || n_groups < 0) return MLF_EINVAL;
    if (K > MLF_MAX_K) return MLF_EUNSUPPORTED;
    if (n_order > 0 && (update_norm_sq == nullptr || order == nullptr)) return MLF_EINVAL;
    if (n_groups > 0 && group_len == nullptr) return MLF_EINVAL;
    if (!(h_norm_sq >= 0.0)) return MLF_EINVAL;
    long long covered = 0;
    for (int j = 0; j < n_groups; ++j) {
        if (group_len[j] < 1 || covered + group_len[j] > n_order) return MLF_EINVAL;
        covered += group_len[j];
    }
    if (covered != n_order) return MLF_EINVAL;
    for (int t = 0; t < n_order; ++t) {
        if (order[t] < 0 || order[t] >= K || !(update_norm_sq[t] >= 0.0)) return MLF_EINVAL;
    }
    const double gamma = static_cast<double>(mu), eta = static_cast<double>(lr);
    // suffix[j] = 1 + gamma + ... + gamma^(S-1-j); the history's coefficient is gamma * suffix[0]
    double suffix[MLF_MAX_K + 1];
    suffix[n_groups] = 0.0;
    for (int j = n_groups - 1; j >= 0; --j) suffix[j] = 1.0 + gamma * suffix[j + 1];
    double total = __builtin_fabs(gamma * suffix[0]) * __builtin_sqrt(h_norm_sq);
    int t = 0;
    for (int j = 0; j < n_groups; ++j) {
        double step = 0.0;
        for (int i = 0; i < group_len[j]; ++i, ++t) {
            const double wt = weights != nullptr ? static_cast<double>(weights[order[t]]) : 1.0;
            step += __builtin_fabs(wt) * __builtin_sqrt(update_norm_sq[t]);
        }
        total += __builtin_fabs(suffix[j]) * __builtin_fabs(eta) * step;
    }
    *bound = total;
    return MLF_OK;
}

// Squared distance of two vectors with the partial sums in `partials` (room for
// capacity + kFinishSlices pairs, capacity >= divergence_partials_capacity()).
// Every partial that is read has been written by this call, so the buffer needs
// no clearing.
static mlf_status divergence_launch(const float *w_server, const float *w_replica, long long n,
                                    double *dist_sq, double *partials, size_t capacity,
                                    hipStream_t s)
{
    const bool aligned16 = reinterpret_cast<uintptr_t>(w_server) % 16 == 0 &&
                           reinterpret_cast<uintptr_t>(w_replica) % 16 == 0;
    const long long n_vec = aligned16 ? n / 4 * 4 : 0;
    const long long per_tile = 64 * kDivUnroll;                      // 128-bit groups per tile
    const long long tiles_v = (n_vec / 4 + per_tile - 1) / per_tile;
    long long tiles_s = (n - n_vec + 63) / 64;
    if (tiles_s > kMaxScalarGroups) tiles_s = kMaxScalarGroups;
    if (tiles_v > 0xffffffffll) return MLF_EUNSUPPORTED;
    const long long groups_v = tiles_v < kDivMaxGroups ? tiles_v : kDivMaxGroups;
    if (static_cast<size_t>(groups_v + tiles_s) > capacity) return MLF_EUNSUPPORTED;
    const unsigned grid = static_cast<unsigned>(groups_v + tiles_s);
    if (grid > 0) {
        if (!launch_kernel(divergence_kernel, dim3(grid), dim3(64), 0, s, w_server, w_replica, n, n_vec,
                           static_cast<unsigned>(tiles_v), static_cast<unsigned>(groups_v), partials)) {
            return MLF_EHIP;
        }
    }
    return finish_norms(partials, grid, capacity, dist_sq, 1, s) ? MLF_OK : MLF_EHIP;
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
                             norms_partials_capacity(n), static_cast<hipStream_t>(stream));
}

// ---------------------------------------------------------------------------
// The divergence for callers that cannot allocate: its partial sums live in a
// file-scope device array instead of a caller's workspace.  Every GPU holds its
// own copy of the array at its own address; the address is looked up once per
// device (hipGetSymbolAddress, with that device current) and kept.  The array's
// name is only ever used in that lookup: host code passes the looked-up pointer.
// ---------------------------------------------------------------------------
constexpr size_t kStaticScratchBytes =
    (divergence_partials_capacity() + kFinishSlices) * 2 * sizeof(double);
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
                             divergence_partials_capacity(), static_cast<hipStream_t>(stream));
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
