// LDA count-delta scatter-add for gfx950 (Sec. 6 of the paper: a worker's LDA
// update is a numerical update to the word-topic count matrix).
//
// Two paths give the same bits (integer addition commutes, so any execution
// order does):
//
// Direct path.  Every workgroup streams a slice of one worker's triple buffer
// and adds the deltas into counts[] with device-scope atomics.  The chip
// retires only a few tens of billions of scattered atomic cache-line operations
// per second, whatever their locality, so this path costs one such operation
// per triple.
//
// Binned path (needs scratch).  Triples are first grouped by the 128 KiB tile
// of counts[] they fall into (a two-level counting sort: 128 fine tiles per
// coarse range, so that every partition step writes contiguous runs; the
// heaviest tiles get a digit of their own at the coarse level and skip the fine
// one).  One workgroup then owns a tile at a time: it accumulates the tile's records
// with LDS atomics into a private 32768-cell image and merges the image into
// counts[] with contiguous 128-bit read-modify-writes (or contiguous atomics
// when a heavy tile is shared by several workgroups).  Global atomic traffic
// drops from one operation per triple to one per touched cache line per
// workgroup, and everything else is streaming.
//
// In both paths the T-entry totals vector, which every triple hits, is kept in
// LDS per workgroup and merged into totals[] once at the end.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "mlfabric.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxLdsTopics = 16384;     // totals privatised in LDS up to 64 KiB

// ---- geometry of the binned path -------------------------------------------
#ifndef MLF_TILE_BITS
#define MLF_TILE_BITS 15
#endif
#ifndef MLF_FINE_BITS
#define MLF_FINE_BITS 7
#endif
#ifndef MLF_ACC_THREADS
#define MLF_ACC_THREADS 1024
#endif
#ifndef MLF_ACC_CHUNK_BITS
#define MLF_ACC_CHUNK_BITS 18
#endif
constexpr int kTileBits = MLF_TILE_BITS;         // log2 of the cells per LDS image
constexpr uint32_t kTileCells = 1u << kTileBits;
constexpr int kFineBits = MLF_FINE_BITS;         // log2 of the fine tiles per coarse range
constexpr uint32_t kFinePerCoarse = 1u << kFineBits;
constexpr uint32_t kMaxCoarse = 256;             // coarse ranges (one counter per lane)
constexpr uint32_t kMaxTiles = 32768;            // tiles a call may span (LDS histogram, plan tables)
constexpr uint32_t kHotWords = kMaxTiles / 32;   // words of the hot-tile bitmap
#ifndef MLF_PART_THREADS
#define MLF_PART_THREADS 1024
#endif
#ifndef MLF_CURSOR_STRIDE
#define MLF_CURSOR_STRIDE 32
#endif
constexpr int kPartThreads = MLF_PART_THREADS;   // lanes of a partition workgroup
#ifndef MLF_PART_ITEMS
#define MLF_PART_ITEMS 8
#endif
constexpr int kPartItems = MLF_PART_ITEMS;       // records per lane in a partition step
constexpr uint32_t kPartTile = kPartThreads * kPartItems;      // records per step
// Output cursors sit this many words apart: every partition step of a range
// bumps the same cursors, and atomics on one cache line are served one by one.
constexpr uint32_t kCursorStride = MLF_CURSOR_STRIDE;
constexpr int kAccThreads = MLF_ACC_THREADS;     // lanes of an accumulate workgroup
constexpr uint32_t kAccChunk = 1u << MLF_ACC_CHUNK_BITS;   // records per accumulate work item
#ifndef MLF_SCAN_UNROLL
#define MLF_SCAN_UNROLL 2
#endif
#ifndef MLF_SCAN_BLOCK
#define MLF_SCAN_BLOCK 1024
#endif
#ifndef MLF_SCAN_WGS
#define MLF_SCAN_WGS 512
#endif
constexpr int kScanBlock = MLF_SCAN_BLOCK;                    // lanes of a first-pass workgroup
constexpr int kScanWorkgroups = MLF_SCAN_WGS;                 // first-pass workgroups of a call, about
constexpr int kScanUnroll = MLF_SCAN_UNROLL;                  // triples per lane and step of the first pass
constexpr int kPlanThreads = 1024;                            // lanes of the one plan workgroup
// The binned path has a fixed cost (six launches, one accumulate workgroup per
// non-empty tile); the direct path is cheaper below about this many triples
// (measured crossovers: 0.25 M triples on a 31-tile matrix, 2 M on 3,052 tiles).
constexpr long long kMinBinnedTriples = 1 << 18;
constexpr long long kMinBinnedTriplesPerTile = 600;

struct SparseArgs {
    const int32_t *triples[MLF_MAX_K];
    long long n_triples[MLF_MAX_K];
    int32_t *counts;
    int32_t *totals;
    int32_t *rejected;
    int V;
    int T;
};

// A triple reduced to what the binned path needs: flat cell index and delta.
struct Record {
    uint32_t cell;
    int32_t delta;
};

// Records travel through the scratch in one of two formats.  LDA deltas are
// almost always +-1, so when every delta of the call lies in
// [-kSmallDeltaLimit, kSmallDeltaLimit) a record is ONE word: between the two
// partition levels the coarse range is implied by where the record lies, which
// leaves kCoarseShift bits of cell index and the rest for the delta; after the
// fine level only the kTileBits cell bits inside the tile are needed.  Otherwise
// (flag raised by the first pass) records are the full 8 bytes.
constexpr int kCoarseShift = kTileBits + kFineBits;
constexpr int32_t kSmallDeltaLimit = 1 << (31 - kCoarseShift);

// The one-word forms of a record.
__device__ __forceinline__ uint32_t pack_tmp(Record r)
{
    return (r.cell & ((1u << kCoarseShift) - 1)) | (static_cast<uint32_t>(r.delta) << kCoarseShift);
}

__device__ __forceinline__ uint32_t pack_sorted(Record r)
{
    return (r.cell & (kTileCells - 1)) | (static_cast<uint32_t>(r.delta) << kTileBits);
}

template <bool WIDE>
__device__ __forceinline__ void store_tmp(void *tmp, uint32_t i, Record r)
{
    if constexpr (WIDE) {
        static_cast<Record *>(tmp)[i] = r;
    } else {
        static_cast<uint32_t *>(tmp)[i] = pack_tmp(r);
    }
}

template <bool WIDE>
__device__ __forceinline__ Record load_tmp(const void *tmp, uint32_t i, uint32_t coarse)
{
    if constexpr (WIDE) {
        return static_cast<const Record *>(tmp)[i];
    } else {
        const uint32_t v = static_cast<const uint32_t *>(tmp)[i];
        return Record{(coarse << kCoarseShift) | (v & ((1u << kCoarseShift) - 1)),
                      static_cast<int32_t>(v) >> kCoarseShift};
    }
}

template <bool WIDE>
__device__ __forceinline__ void store_sorted(void *sorted, uint32_t i, Record r)
{
    if constexpr (WIDE) {
        static_cast<Record *>(sorted)[i] = r;
    } else {
        static_cast<uint32_t *>(sorted)[i] = pack_sorted(r);
    }
}

// Returns the cell index inside the tile and the delta.
template <bool WIDE>
__device__ __forceinline__ Record load_sorted(const void *sorted, uint32_t i)
{
    if constexpr (WIDE) {
        const Record r = static_cast<const Record *>(sorted)[i];
        return Record{r.cell & (kTileCells - 1), r.delta};
    } else {
        const uint32_t v = static_cast<const uint32_t *>(sorted)[i];
        return Record{v & (kTileCells - 1), static_cast<int32_t>(v) >> kTileBits};
    }
}

// Control block of the binned path, carved out of the caller's scratch.
struct BinPlan {
    uint32_t *hist;               // [n_tiles]   records per tile            (zeroed)
    uint32_t *coarse_cursor;      // [kMaxCoarse * kCursorStride] records placed so far per digit of the
                                  //                             coarse level (zeroed)
    uint32_t *fine_cursor;        // [n_tiles * kCursorStride]  records placed so far (zeroed)
    uint32_t *tile_start;         // [n_tiles+1] exclusive scan of hist
    uint32_t *coarse_part_start;  // [n_coarse+1] partition steps before each coarse range
    uint32_t *chunk_start;        // [n_tiles+1] accumulate work items of the tiles that are not hot,
                                  //             before each tile
    uint32_t *hot_chunk_start;    // [kMaxCoarse+1] accumulate work items before each hot tile; the hot
                                  //             tiles' items come first in the launch
    uint32_t *hot_tile;           // [kMaxCoarse] tile of each hot digit
    uint32_t *tmp_start;          // [n_coarse+1] first record of each coarse range in tmp
    uint32_t *digit_start;        // [kMaxCoarse] first output index of each digit of the coarse level:
                                  //              in tmp for a coarse range, in sorted for a hot tile
    uint32_t *hot_bits;           // [kHotWords] bit b set = tile b is hot
    uint32_t *hot_before;         // [kHotWords] hot tiles before the first tile of each word
    uint32_t *wide_flag;          // [1] non-zero: some delta needs the 8-byte record (zeroed)
    void *tmp;                    // [n] records grouped by coarse range
    void *sorted;                 // [n] records grouped by tile
    uint32_t n_tiles;
    uint32_t n_coarse;
    unsigned long long n_cells;   // V * T
};

__device__ __forceinline__ void add_relaxed(int32_t *p, int32_t v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t fetch_add_relaxed(uint32_t *p, uint32_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ uint32_t lds_fetch_add(uint32_t *p, uint32_t v)
{
    return __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ void lds_add(int32_t *p, int32_t v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Number of lanes below the caller whose bit is set in `mask`.
__device__ __forceinline__ uint32_t lanes_below(unsigned long long mask)
{
    return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                     __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), 0u));
}

// The value of lane `lane` (the same for all lanes of the wavefront) in every
// lane: a register read, where a shuffle would go through the LDS pipeline.
__device__ __forceinline__ uint32_t broadcast(uint32_t v, int lane)
{
    return static_cast<uint32_t>(
        __builtin_amdgcn_readlane(static_cast<int>(v), __builtin_amdgcn_readfirstlane(lane)));
}

// counter[bin] += 1 for every live lane, returning to each the value it would
// have seen had the lanes gone one by one (its rank in the bin).  Skewed data
// puts most lanes of a wavefront into one bin, and LDS atomics on one address
// are served one lane at a time; so the lanes that share the bin of the first
// live lane are counted with a ballot and added by a single atomic, and only
// the others go one by one.  Must be called by whole wavefronts.
__device__ __forceinline__ uint32_t wave_rank(uint32_t *counter, uint32_t bin, bool live)
{
    const unsigned long long live_mask = __ballot(live);
    if (live_mask == 0) return 0;                                   // uniform
    const int leader = __ffsll(static_cast<long long>(live_mask)) - 1;
    const uint32_t lead_bin = broadcast(bin, leader);
    const bool grouped = live && bin == lead_bin;
    const unsigned long long group = __ballot(grouped);
    uint32_t base = 0;
    if (static_cast<int>(threadIdx.x & 63) == leader) {
        // (indexed by the lane's own bin, which equals lead_bin here)
        base = lds_fetch_add(&counter[bin], static_cast<uint32_t>(__popcll(group)));
    }
    base = broadcast(base, leader);
    if (grouped) return base + lanes_below(group);
    return live ? lds_fetch_add(&counter[bin], 1u) : 0u;
}

// counter[bin] += 1 for every active lane, with the same grouping of the lanes
// that share the first active lane's bin; no value is returned.
__device__ __forceinline__ void wave_count(uint32_t *counter, uint32_t bin)
{
    const unsigned long long active = __ballot(true);
    const int leader = __ffsll(static_cast<long long>(active)) - 1;
    const uint32_t lead_bin = broadcast(bin, leader);
    const bool grouped = bin == lead_bin;
    const unsigned long long group = __ballot(grouped);
    if (static_cast<int>(threadIdx.x & 63) == leader) {
        lds_fetch_add(&counter[lead_bin], static_cast<uint32_t>(__popcll(group)));
    } else if (!grouped) {
        lds_fetch_add(&counter[bin], 1u);
    }
}

// Reads triple r of a buffer (read once: streaming loads) and tells whether
// its word and topic are in range.
__device__ __forceinline__ bool load_triple(const int32_t *tr, long long r, int V, int T,
                                            int &word, int &topic, int &delta)
{
    word = __builtin_nontemporal_load(tr + 3 * r);
    topic = __builtin_nontemporal_load(tr + 3 * r + 1);
    delta = __builtin_nontemporal_load(tr + 3 * r + 2);
    return static_cast<unsigned>(word) < static_cast<unsigned>(V) &&
           static_cast<unsigned>(topic) < static_cast<unsigned>(T);
}

// First pass over the triples; blockIdx.y = worker buffer, blockIdx.x = share
// of that buffer.  BINNED = false: the direct path (counts[] updated here).
// BINNED = true: only the per-tile histogram is built.  Both keep the totals in
// LDS and count the rejected triples.
// LDS: [T totals if LDS_TOTALS][n_tiles histogram if BINNED], dynamic up to
// 64 KiB; BIG = a static array instead, for histograms of up to kMaxTiles tiles
// with up to kBigTopics totals.
constexpr int kBigTopics = 4096;

template <bool BINNED, bool LDS_TOTALS, bool BIG = false>
__global__ __launch_bounds__(kScanBlock) void scan_triples_kernel(const SparseArgs a,
                                                                const BinPlan plan)
{
    extern __shared__ int32_t dynamic_lds[];
    __shared__ int32_t static_lds[BIG ? kMaxTiles + kBigTopics : 1];
    int32_t *lds = BIG ? static_lds : dynamic_lds;
    const int T = a.T;
    const bool want_totals = a.totals != nullptr;
    int32_t *lds_totals = lds;
    uint32_t *lds_hist = reinterpret_cast<uint32_t *>(lds + (LDS_TOTALS ? T : 0));
    if constexpr (LDS_TOTALS) {
        for (int t = threadIdx.x; t < T; t += kScanBlock) lds_totals[t] = 0;
    }
    if constexpr (BINNED) {
        for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kScanBlock) lds_hist[b] = 0;
    }
    if constexpr (LDS_TOTALS || BINNED) __syncthreads();

    const int k = blockIdx.y;
    const int32_t *tr = a.triples[k];
    const long long m = a.n_triples[k];
    // Each workgroup streams one contiguous share of the buffer (rather than
    // striding over it with the others), so that at any moment the workgroups
    // of a launch read from places spread over all the buffers.
    constexpr long long kStep = static_cast<long long>(kScanBlock) * kScanUnroll;
    const long long share = ((m + gridDim.x - 1) / gridDim.x + kStep - 1) / kStep * kStep;
    const long long begin = min(static_cast<long long>(blockIdx.x) * share, m);
    const long long end = min(begin + share, m);
    int n_bad = 0;
    bool wide = false;
    // kScanUnroll triples per lane and step, all loaded before the first is used.
    for (long long r0 = begin + threadIdx.x; r0 < end; r0 += kStep) {
        int word[kScanUnroll], topic[kScanUnroll], delta[kScanUnroll];
        bool there[kScanUnroll], good[kScanUnroll];
#pragma unroll
        for (int u = 0; u < kScanUnroll; ++u) {
            const long long r = r0 + u * kScanBlock;
            there[u] = r < end;
            word[u] = topic[u] = delta[u] = 0;
            good[u] = there[u] && load_triple(tr, r, a.V, T, word[u], topic[u], delta[u]);
        }
#pragma unroll
        for (int u = 0; u < kScanUnroll; ++u) {
            if (!there[u]) continue;
            if (!good[u]) {
                ++n_bad;
                continue;
            }
            const long long cell = static_cast<long long>(word[u]) * T + topic[u];
            if constexpr (BINNED) {
                wide = wide || delta[u] < -kSmallDeltaLimit || delta[u] >= kSmallDeltaLimit;
                wave_count(lds_hist, static_cast<uint32_t>(cell) >> kTileBits);
            } else {
                add_relaxed(a.counts + cell, delta[u]);
            }
            if (want_totals) {
                if constexpr (LDS_TOTALS) {
                    lds_add(&lds_totals[topic[u]], delta[u]);
                } else {
                    add_relaxed(a.totals + topic[u], delta[u]);
                }
            }
        }
    }

    if constexpr (LDS_TOTALS || BINNED) __syncthreads();
    if constexpr (LDS_TOTALS) {
        if (want_totals) {
            for (int t = threadIdx.x; t < T; t += kScanBlock) {
                const int32_t v = lds_totals[t];
                if (v != 0) add_relaxed(a.totals + t, v);
            }
        }
    }
    if constexpr (BINNED) {
        for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kScanBlock) {
            const uint32_t v = lds_hist[b];
            if (v != 0) fetch_add_relaxed(plan.hist + b, v);
        }
        // One lane per wavefront raises the flag if any lane met a large delta.
        if (__ballot(wide) != 0 && (threadIdx.x & 63) == 0) {
            __hip_atomic_fetch_or(plan.wide_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    if (a.rejected != nullptr) {
        // Wavefront sum of the per-lane reject counts, one atomic per wavefront.
        for (int off = 32; off > 0; off >>= 1) n_bad += __shfl_down(n_bad, off, 64);
        if ((threadIdx.x & 63) == 0 && n_bad != 0) add_relaxed(a.rejected, n_bad);
    }
}

// Clears the counters of the binned path (a kernel rather than a memset so that
// the whole call can be recorded into a graph).
__global__ __launch_bounds__(kThreads) void clear_kernel(uint32_t *p, uint32_t n)
{
    const uint32_t i = blockIdx.x * kThreads + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Exclusive prefix sums of N values per lane over the kPlanThreads lanes of
// the workgroup: shuffles inside each wavefront, then the wavefront totals
// through LDS.  excl[k] = sum of v[k] over the lanes before this one, total[k] =
// sum over all lanes.  Two barriers; `wave_sums` is reused by the next call.
constexpr int kPlanWaves = kPlanThreads / 64;

template <int N>
__device__ __forceinline__ void block_scan(const uint32_t (&v)[N], uint32_t (&excl)[N],
                                           uint32_t (&total)[N], uint32_t (*wave_sums)[kPlanWaves])
{
    const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    uint32_t incl[N];
#pragma unroll
    for (int k = 0; k < N; ++k) incl[k] = v[k];
    for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
        for (int k = 0; k < N; ++k) {
            const uint32_t up = __shfl_up(incl[k], off, 64);
            if (lane >= static_cast<uint32_t>(off)) incl[k] += up;
        }
    }
    if (lane == 63) {
#pragma unroll
        for (int k = 0; k < N; ++k) wave_sums[k][wave] = incl[k];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < N; ++k) {
        uint32_t before = 0, all = 0;
#pragma unroll
        for (int w = 0; w < kPlanWaves; ++w) {
            const uint32_t t = wave_sums[k][w];
            before += static_cast<uint32_t>(w) < wave ? t : 0u;
            all += t;
        }
        excl[k] = before + incl[k] - v[k];
        total[k] = all;
    }
    __syncthreads();
}

// One workgroup: turns the tile histogram into the offsets every later step uses.
//
// Heavy tiles skip the fine level.  The coarse level has kMaxCoarse digits and
// needs n_coarse of them for the coarse ranges; each spare digit is given to one
// of the heaviest tiles ("hot"), whose records the coarse level then writes
// straight to their final place in `sorted`.  Under a Zipf law a few hundred
// tiles hold most of the records, so most records are moved once instead of
// twice.  The hot tiles are those with at least `threshold` records, the
// smallest power-of-two fraction of the total that leaves no more hot tiles
// than spare digits.  They are published as a bitmap plus, per bitmap word, the
// number of hot tiles before it, so that a lane finds the digit of a tile with
// one LDS read and a population count.
//
// Lane i looks after the tiles i, i + kPlanThreads, ... (one per round); the
// record counts are kept in LDS, and every table over the tiles is a running
// block scan over the rounds.  (The rounds are loops, not unrolled: the kernel
// runs once per call, and straight-line code would be fetched from memory once.)
#ifndef MLF_HOT_SHIFTS
#define MLF_HOT_SHIFTS 24
#endif
constexpr int kHotShifts = MLF_HOT_SHIFTS;     // a hot tile holds at least total >> (kHotShifts - 1) records

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const BinPlan plan)
{
    static_assert(kMaxCoarse <= kPlanThreads, "the tables over coarse digits take one round");
    __shared__ uint32_t wave_sums[3][kPlanWaves];
    __shared__ uint32_t tiles_at_least[kHotShifts];
    __shared__ uint32_t hot_in_range[kMaxCoarse];     // hot records per coarse range
    __shared__ uint32_t s_threshold;
    __shared__ uint32_t h[kMaxTiles];                 // records per tile
    const uint32_t n_tiles = plan.n_tiles;
    const uint32_t n_coarse = plan.n_coarse;
    const uint32_t lane = threadIdx.x & 63;

    if (threadIdx.x < kHotShifts) tiles_at_least[threadIdx.x] = 0;
    if (threadIdx.x < kMaxCoarse) hot_in_range[threadIdx.x] = 0;

    // tile_start: exclusive scan of the histogram.
    uint32_t total = 0;
#pragma unroll 1
    for (uint32_t base = 0; base < n_tiles; base += kPlanThreads) {
        const uint32_t b = base + threadIdx.x;
        const uint32_t v[1] = {b < n_tiles ? plan.hist[b] : 0u};
        h[b] = v[0];
        uint32_t e[1], t[1];
        block_scan<1>(v, e, t, wave_sums);
        if (b < n_tiles) plan.tile_start[b] = total + e[0];
        total += t[0];
    }
    if (threadIdx.x == 0) plan.tile_start[n_tiles] = total;

    // Threshold of the hot tiles.
#pragma unroll 1
    for (uint32_t base = 0; base < n_tiles; base += kPlanThreads) {
        const uint32_t mine = h[base + threadIdx.x];
#pragma unroll 1
        for (int j = 0; j < kHotShifts; ++j) {
            const unsigned long long heavy = __ballot(mine != 0 && mine >= (total >> j));
            if (lane == 0 && heavy != 0) {
                lds_fetch_add(&tiles_at_least[j], static_cast<uint32_t>(__popcll(heavy)));
            }
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t spare = kMaxCoarse - n_coarse;
        uint32_t threshold = 0xffffffffu;                    // no hot tile
        for (int j = 0; j < kHotShifts; ++j) {
            if (tiles_at_least[j] <= spare && (total >> j) >= 1) threshold = total >> j;
        }
        s_threshold = threshold;
    }
    __syncthreads();
    const uint32_t threshold = s_threshold;

    // Hot tiles: bitmap (the words that cover the call's tiles), digit of each
    // (its rank among the hot tiles), hot records per coarse range; and the
    // accumulate work items (kAccChunk records each) of the tiles that are not hot.
    uint32_t n_hot = 0, n_items = 0;
#pragma unroll 1
    for (uint32_t base = 0; base < n_tiles; base += kPlanThreads) {
        const uint32_t b = base + threadIdx.x;
        const uint32_t mine = h[b];
        const bool hot = mine != 0 && mine >= threshold;
        const unsigned long long mask = __ballot(hot);
        if (lane == 0) {
            plan.hot_bits[b >> 5] = static_cast<uint32_t>(mask);
            plan.hot_bits[(b >> 5) + 1] = static_cast<uint32_t>(mask >> 32);
        }
        const uint32_t v[2] = {hot ? 1u : 0u, hot ? 0u : (mine + kAccChunk - 1) / kAccChunk};
        uint32_t e[2], t[2];
        block_scan<2>(v, e, t, wave_sums);
        const uint32_t slot = n_hot + e[0];
        if ((threadIdx.x & 31) == 0) plan.hot_before[b >> 5] = slot;
        if (hot) {
            plan.hot_tile[slot] = b;
            plan.digit_start[n_coarse + slot] = plan.tile_start[b];      // this lane wrote it
            lds_fetch_add(&hot_in_range[b >> kFineBits], mine);
        }
        if (b < n_tiles) plan.chunk_start[b] = n_items + e[1];
        n_hot += t[0];
        n_items += t[1];
    }
    if (threadIdx.x == 0) {
        plan.hot_before[kHotWords] = n_hot;
        plan.chunk_start[n_tiles] = n_items;
    }
    __syncthreads();
    __threadfence_block();

    // Per coarse range: the records that still go through the fine level and
    // their partition steps (kPartTile records each); per hot digit: the
    // accumulate work items of its tile, which come first in that launch so
    // that the long ones start early.
    {
        const uint32_t c = threadIdx.x;
        uint32_t cold = 0;
        if (c < n_coarse) {
            const uint32_t lo = c << kFineBits;
            const uint32_t hi = min(lo + kFinePerCoarse, n_tiles);
            cold = plan.tile_start[hi] - plan.tile_start[lo] - hot_in_range[c];
        }
        uint32_t hot_items = 0;
        if (c < n_hot) hot_items = (h[plan.hot_tile[c]] + kAccChunk - 1) / kAccChunk;
        const uint32_t v[3] = {cold, (cold + kPartTile - 1) / kPartTile, hot_items};
        uint32_t e[3], t[3];
        block_scan<3>(v, e, t, wave_sums);
        if (c < n_coarse) {
            plan.tmp_start[c] = e[0];
            plan.digit_start[c] = e[0];
            plan.coarse_part_start[c] = e[1];
        }
        if (c == n_coarse) {
            plan.tmp_start[c] = t[0];
            plan.coarse_part_start[c] = t[1];
        }
        if (c <= kMaxCoarse) plan.hot_chunk_start[c] = c < kMaxCoarse ? e[2] : t[2];
    }
}

// Largest index i in [0, n) with start[i] <= g, for a non-decreasing start[] with
// start[0] = 0 and g < start[n].  Called by one whole wavefront: its 64 lanes
// probe 64 evenly spaced entries per round, so that 4,096 entries take two
// rounds of dependent loads where a binary search by one lane takes twelve.
__device__ __forceinline__ uint32_t owner_of(const uint32_t *start, uint32_t n, uint32_t g)
{
    const uint32_t lane = threadIdx.x & 63;
    uint32_t lo = 0, hi = n;                       // the answer is in [lo, hi)
    while (hi - lo > 1) {
        const uint32_t step = (hi - lo + 63) / 64;
        const uint32_t idx = lo + lane * step;
        // start[lo] <= g always, so lane 0 votes yes; the votes are a prefix of the lanes.
        const unsigned long long yes = __ballot(idx < hi && start[idx] <= g);
        const uint32_t last = static_cast<uint32_t>(__popcll(yes)) - 1;
        lo += last * step;
        hi = min(lo + step, hi);
    }
    return lo;
}

// One partition step of a workgroup: up to kPartTile records held in registers
// are grouped by digit (< kMaxCoarse) in LDS and written out so that the records
// of one digit form one contiguous run at the place reserved for them.
//   rec[i], live[i]  the lane's records and whether each exists
//   digit_of(cell)   digit of a record
//   reserve(d, n)    output index where this step's n records of digit d go
// Eight-byte records (WIDE) are staged as they are and placed when they are
// written out:
//   emit(d, i, r)    writes record r of digit d at output index i
// One-word records are packed and given their output index when they are
// staged, so that writing them out is a copy:
//   pack(d, r)       the word to store for record r of digit d; bit 31 of the
//                    result's `where` selects the output array
//   copy(where, w)   stores word w at output index (where & 0x7fffffff)
struct Staged {
    uint32_t word;
    uint32_t where;
};

struct PartitionLds {
    union {
        Record wide[kPartTile];
        Staged narrow[kPartTile];
    } stage;
    uint32_t count[kMaxCoarse];
    uint32_t offset[kMaxCoarse];
    uint32_t dest[kMaxCoarse];
    uint32_t total;
};

template <bool WIDE, typename DigitOf, typename Reserve, typename Emit, typename Pack, typename Copy>
__device__ __forceinline__ void partition_step(PartitionLds &s, const Record (&rec)[kPartItems],
                                               const bool (&live)[kPartItems], DigitOf digit_of,
                                               Reserve reserve, Emit emit, Pack pack, Copy copy)
{
    static_assert(kMaxCoarse == 256 && kPartThreads >= 256, "one wavefront scans 4 digits per lane");
    uint32_t dig[kPartItems], rank[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        dig[i] = live[i] ? digit_of(rec[i].cell) : 0u;
        rank[i] = wave_rank(s.count, dig[i], live[i]);
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        // Exclusive scan of the 256 digit counts by one wavefront: 4 per lane,
        // then a shuffle scan of the lane sums.
        const uint32_t lane = threadIdx.x;
        uint32_t c[4];
        uint32_t sum = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            c[k] = s.count[4 * lane + k];
            sum += c[k];
        }
        uint32_t incl = sum;
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t up = __shfl_up(incl, off, 64);
            if (lane >= static_cast<uint32_t>(off)) incl += up;
        }
        uint32_t run = incl - sum;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            s.offset[4 * lane + k] = run;
            run += c[k];
        }
        if (lane == 63) s.total = incl;
    }
    if (threadIdx.x < kMaxCoarse) {
        const uint32_t mine = s.count[threadIdx.x];
        if (mine != 0) s.dest[threadIdx.x] = reserve(threadIdx.x, mine);
    }
    __syncthreads();
    if constexpr (WIDE) {
#pragma unroll
        for (int i = 0; i < kPartItems; ++i) {
            if (live[i]) s.stage.wide[s.offset[dig[i]] + rank[i]] = rec[i];
        }
        __syncthreads();
        const uint32_t total = s.total;
        for (uint32_t i = threadIdx.x; i < total; i += kPartThreads) {
            const Record r = s.stage.wide[i];
            const uint32_t d = digit_of(r.cell);
            emit(d, s.dest[d] + (i - s.offset[d]), r);
        }
    } else {
#pragma unroll
        for (int i = 0; i < kPartItems; ++i) {
            if (live[i]) {
                Staged e = pack(dig[i], rec[i]);
                e.where |= s.dest[dig[i]] + rank[i];
                s.stage.narrow[s.offset[dig[i]] + rank[i]] = e;
            }
        }
        __syncthreads();
        const uint32_t total = s.total;
        for (uint32_t i = threadIdx.x; i < total; i += kPartThreads) {
            const Staged e = s.stage.narrow[i];
            copy(e.where, e.word);
        }
    }
}

// Coarse partition: blockIdx.y = worker buffer, blockIdx.x = step within it.
// Valid triples become records: those of hot tiles go to their final place in
// plan.sorted, the others to plan.tmp, grouped by coarse range.
struct HotLds {
    uint2 word[kHotWords];      // x = bitmap word, y = hot tiles before it: one 64-bit read per lookup
};

template <bool WIDE>
__device__ __forceinline__ void coarse_partition_body(PartitionLds &s, HotLds &hot,
                                                      const SparseArgs &a, const BinPlan &plan)
{
    const int32_t *tr = a.triples[blockIdx.y];
    const long long m = a.n_triples[blockIdx.y];
    const long long base = static_cast<long long>(blockIdx.x) * kPartTile;
    if (base >= m) return;                               // uniform for the workgroup
    Record rec[kPartItems];
    bool live[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        const long long r = base + i * kPartThreads + threadIdx.x;
        int word = 0, topic = 0, delta = 0;
        live[i] = r < m && load_triple(tr, r, a.V, a.T, word, topic, delta);
        rec[i].cell = static_cast<uint32_t>(static_cast<long long>(word) * a.T + topic);
        rec[i].delta = delta;
    }
    // The hot-tile bitmap and the digit counters, while the triples are in flight.
    static_assert(kHotWords <= kPartThreads && kMaxCoarse <= kPartThreads, "one word per lane");
    if (threadIdx.x < (plan.n_tiles + 31) / 32) {       // the words that cover the call's tiles
        hot.word[threadIdx.x] = make_uint2(plan.hot_bits[threadIdx.x], plan.hot_before[threadIdx.x]);
    }
    if (threadIdx.x < kMaxCoarse) s.count[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t n_coarse = plan.n_coarse;
    const HotLds *h = &hot;
    uint32_t *tmp_words = static_cast<uint32_t *>(plan.tmp);
    uint32_t *sorted_words = static_cast<uint32_t *>(plan.sorted);
    partition_step<WIDE>(
        s, rec, live,
        [=](uint32_t cell) {
            const uint32_t tile = cell >> kTileBits;
            const uint2 entry = h->word[tile >> 5];
            const uint32_t bit = tile & 31;
            const uint32_t hot_digit =
                n_coarse + entry.y + static_cast<uint32_t>(__popc(entry.x & ((1u << bit) - 1u)));
            return ((entry.x >> bit) & 1u) != 0 ? hot_digit : tile >> kFineBits;
        },
        [=](uint32_t d, uint32_t n) {
            return plan.digit_start[d] + fetch_add_relaxed(plan.coarse_cursor + d * kCursorStride, n);
        },
        [=](uint32_t d, uint32_t i, Record r) {
            if (d < n_coarse) {
                store_tmp<WIDE>(plan.tmp, i, r);
            } else {
                store_sorted<WIDE>(plan.sorted, i, r);
            }
        },
        [=](uint32_t d, Record r) {
            return d < n_coarse ? Staged{pack_tmp(r), 0u} : Staged{pack_sorted(r), 0x80000000u};
        },
        [=](uint32_t where, uint32_t word) {
            uint32_t *out = (where >> 31) != 0 ? sorted_words : tmp_words;
            out[where & 0x7fffffffu] = word;
        });
}

// The record format of the call, the same for every lane (scalar register).
__device__ __forceinline__ bool wide_records(const BinPlan &plan)
{
    return __builtin_amdgcn_readfirstlane(static_cast<int>(*plan.wide_flag)) != 0;
}

__global__ __launch_bounds__(kPartThreads) void coarse_partition_kernel(const SparseArgs a,
                                                                    const BinPlan plan)
{
    __shared__ PartitionLds s;
    __shared__ HotLds hot;
    if (wide_records(plan)) {
        coarse_partition_body<true>(s, hot, a, plan);
    } else {
        coarse_partition_body<false>(s, hot, a, plan);
    }
}

// Fine partition: workgroup g takes one step of one coarse range of plan.tmp
// and writes its records to plan.sorted, grouped by tile.
template <bool WIDE>
__device__ __forceinline__ void fine_partition_body(PartitionLds &s, const BinPlan &plan, uint32_t g,
                                                    uint32_t c)
{
    const uint32_t first_tile = c << kFineBits;
    const uint32_t begin = plan.tmp_start[c] + (g - plan.coarse_part_start[c]) * kPartTile;
    const uint32_t end = min(begin + kPartTile, plan.tmp_start[c + 1]);
    Record rec[kPartItems];
    bool live[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        const uint32_t r = begin + i * kPartThreads + threadIdx.x;
        live[i] = r < end;
        rec[i] = live[i] ? load_tmp<WIDE>(plan.tmp, r, c) : Record{0u, 0};
    }
    if (threadIdx.x < kMaxCoarse) s.count[threadIdx.x] = 0;
    __syncthreads();
    uint32_t *sorted_words = static_cast<uint32_t *>(plan.sorted);
    partition_step<WIDE>(
        s, rec, live, [](uint32_t cell) { return (cell >> kTileBits) & (kFinePerCoarse - 1); },
        [=](uint32_t f, uint32_t n) {
            const uint32_t tile = first_tile + f;
            return plan.tile_start[tile] + fetch_add_relaxed(plan.fine_cursor + tile * kCursorStride, n);
        },
        [=](uint32_t, uint32_t i, Record r) { store_sorted<WIDE>(plan.sorted, i, r); },
        [](uint32_t, Record r) { return Staged{pack_sorted(r), 0u}; },
        [=](uint32_t where, uint32_t word) { sorted_words[where] = word; });
}

__global__ __launch_bounds__(kPartThreads) void fine_partition_kernel(const BinPlan plan)
{
    __shared__ PartitionLds s;
    __shared__ uint32_t s_coarse;
    const uint32_t g = blockIdx.x;
    if (g >= plan.coarse_part_start[plan.n_coarse]) return;   // uniform
    if (threadIdx.x < 64) {
        const uint32_t c = owner_of(plan.coarse_part_start, plan.n_coarse, g);
        if (threadIdx.x == 0) s_coarse = c;
    }
    __syncthreads();
    const uint32_t c = s_coarse;
    if (wide_records(plan)) {
        fine_partition_body<true>(s, plan, g, c);
    } else {
        fine_partition_body<false>(s, plan, g, c);
    }
}

// Accumulate: workgroup g takes up to kAccChunk records of one tile, sums them
// into a private LDS image of the tile and merges the image into counts[].
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
#ifndef MLF_ACC_UNROLL
#define MLF_ACC_UNROLL 4
#endif
constexpr int kAccUnroll = MLF_ACC_UNROLL;       // 128-bit record loads in flight per lane

// Adds the records [begin, end) of one tile into its LDS image.  The records
// are read with 128-bit loads (4 narrow or 2 wide records each), kAccUnroll of
// them in flight per lane; the few records before the first and after the last
// aligned group go one by one.
template <bool WIDE>
__device__ __forceinline__ void accumulate_records(int32_t *image, const void *__restrict__ sorted,
                                                   uint32_t begin, uint32_t end)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr uint32_t kPer = WIDE ? 2 : 4;
    const uint32_t first = min((begin + kPer - 1) / kPer * kPer, end);
    const uint32_t last = max(first, end / kPer * kPer);
    auto add_one = [&](uint32_t r) {
        const Record rec = load_sorted<WIDE>(sorted, r);
        lds_add(&image[rec.cell], rec.delta);
    };
    if (threadIdx.x < first - begin) add_one(begin + threadIdx.x);
    if (threadIdx.x < end - last) add_one(last + threadIdx.x);

    const u32x4 *groups = static_cast<const u32x4 *>(sorted);
    const uint32_t g_end = last / kPer;
    for (uint32_t g0 = first / kPer + threadIdx.x; g0 < g_end; g0 += kAccThreads * kAccUnroll) {
        u32x4 x[kAccUnroll];
#pragma unroll
        for (int u = 0; u < kAccUnroll; ++u) {
            const uint32_t g = g0 + u * kAccThreads;
            x[u] = g < g_end ? groups[g] : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kAccUnroll; ++u) {
            if (g0 + u * kAccThreads >= g_end) continue;
            if constexpr (WIDE) {
                lds_add(&image[x[u].x & (kTileCells - 1)], static_cast<int32_t>(x[u].y));
                lds_add(&image[x[u].z & (kTileCells - 1)], static_cast<int32_t>(x[u].w));
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t v = x[u][j];
                    lds_add(&image[v & (kTileCells - 1)], static_cast<int32_t>(v) >> kTileBits);
                }
            }
        }
    }
}

__global__ __launch_bounds__(kAccThreads) void accumulate_kernel(int32_t *__restrict__ counts,
                                                                 const BinPlan plan)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr int kGroupsPerLane = kTileCells / 4 / kAccThreads;
    __shared__ __attribute__((aligned(16))) int32_t image[kTileCells];
    __shared__ uint32_t s_tile;
    __shared__ uint32_t s_first;                  // work items before this tile's, in its list
    const uint32_t n_hot_items = plan.hot_chunk_start[kMaxCoarse];
    if (blockIdx.x >= n_hot_items + plan.chunk_start[plan.n_tiles]) return;      // uniform
    const bool hot = blockIdx.x < n_hot_items;
    const uint32_t g = hot ? blockIdx.x : blockIdx.x - n_hot_items;               // item in its list
    const uint32_t *start = hot ? plan.hot_chunk_start : plan.chunk_start;
    if (threadIdx.x < 64) {
        const uint32_t i = owner_of(start, hot ? kMaxCoarse : plan.n_tiles, g);
        if (threadIdx.x == 0) {
            s_tile = hot ? plan.hot_tile[i] : i;
            s_first = i;
        }
    }
    i32x4 *image4 = reinterpret_cast<i32x4 *>(image);
#pragma unroll
    for (int k = 0; k < kGroupsPerLane; ++k) image4[k * kAccThreads + threadIdx.x] = i32x4{0, 0, 0, 0};
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint32_t chunks = start[s_first + 1] - start[s_first];
    const uint32_t begin = plan.tile_start[tile] + (g - start[s_first]) * kAccChunk;
    const uint32_t end = min(begin + kAccChunk, plan.tile_start[tile + 1]);
    if (wide_records(plan)) {
        accumulate_records<true>(image, plan.sorted, begin, end);
    } else {
        accumulate_records<false>(image, plan.sorted, begin, end);
    }
    __syncthreads();
    const unsigned long long base = static_cast<unsigned long long>(tile) << kTileBits;
    const unsigned long long left = plan.n_cells - base;
    const uint32_t cells = left < kTileCells ? static_cast<uint32_t>(left) : kTileCells;
    int32_t *__restrict__ dst = counts + base;
    // 128-bit groups where the destination allows it, single cells otherwise.
    const uint32_t groups = reinterpret_cast<uintptr_t>(dst) % 16 == 0 ? cells / 4 : 0;
    if (chunks == 1) {
        // This workgroup is the only writer of the tile: plain read-modify-write
        // (int32 addition wraps; done on unsigned values).  All loads of a lane
        // are issued before its first store, so their latencies overlap.
        u32x4 *dst4 = reinterpret_cast<u32x4 *>(dst);
        u32x4 add[kGroupsPerLane], old[kGroupsPerLane];
        bool touch[kGroupsPerLane];
#pragma unroll
        for (int k = 0; k < kGroupsPerLane; ++k) {
            const uint32_t i = k * kAccThreads + threadIdx.x;
            add[k] = __builtin_bit_cast(u32x4, image4[i]);
            touch[k] = i < groups && (add[k].x | add[k].y | add[k].z | add[k].w) != 0;
            old[k] = touch[k] ? dst4[i] : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int k = 0; k < kGroupsPerLane; ++k) {
            if (touch[k]) dst4[k * kAccThreads + threadIdx.x] = old[k] + add[k];
        }
        for (uint32_t i = groups * 4 + threadIdx.x; i < cells; i += kAccThreads) {
            const int32_t v = image[i];
            if (v != 0) dst[i] = static_cast<int32_t>(static_cast<uint32_t>(dst[i]) + static_cast<uint32_t>(v));
        }
    } else {
        // Shared tile: lane i adds cell i, so a wavefront's atomics are contiguous.
        for (uint32_t i = threadIdx.x; i < cells; i += kAccThreads) {
            const int32_t v = image[i];
            if (v != 0) add_relaxed(dst + i, v);
        }
    }
}

// ---------------------------------------------------------------------------
// The same LDA update exchanged as dense V x T delta matrices (Sec. 6 of the
// paper): counts += sum over the workers, totals += its column sums.  A
// streaming kernel like the dense float path: every delta matrix is read once
// with 128-bit loads, counts is read and written once, each cell is owned by
// one lane (no atomics on counts); the column sums go through the per-workgroup
// LDS copy of the totals.
// ---------------------------------------------------------------------------
#ifndef MLF_DELTA_CHUNK
#define MLF_DELTA_CHUNK 8
#endif
constexpr int kDeltaChunk = MLF_DELTA_CHUNK;   // delta matrices whose loads are in flight together
#ifndef MLF_DELTA_VPT
#define MLF_DELTA_VPT 2
#endif
constexpr int kDeltaVpt = MLF_DELTA_VPT;       // 128-bit groups per lane and step
#ifndef MLF_DELTA_THREADS
#define MLF_DELTA_THREADS 1024
#endif
constexpr int kDeltaThreads = MLF_DELTA_THREADS;   // lanes of a workgroup
#ifndef MLF_DELTA_MAX_GRID
#define MLF_DELTA_MAX_GRID 2048
#endif
constexpr unsigned kDeltaMaxGrid = MLF_DELTA_MAX_GRID;

struct DeltaArgs {
    const int32_t *delta[MLF_MAX_K];
    int32_t *counts;
    int32_t *totals;
    unsigned long long n_cells;     // V * T
    unsigned long long n_vec;       // leading cells on the 128-bit path (0 if unaligned)
    int K;
    int T;
};

template <bool LDS_TOTALS>
__device__ __forceinline__ void add_to_total(const DeltaArgs &a, int32_t *lds_totals, uint32_t col,
                                             uint32_t v)
{
    if (v == 0 || a.totals == nullptr) return;
    if constexpr (LDS_TOTALS) {
        lds_add(&lds_totals[col], static_cast<int32_t>(v));
    } else {
        add_relaxed(a.totals + col, static_cast<int32_t>(v));
    }
}

template <bool LDS_TOTALS>
__global__ __launch_bounds__(kDeltaThreads) void dense_delta_kernel(const DeltaArgs a)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    extern __shared__ int32_t lds_totals[];
    const uint32_t T = static_cast<uint32_t>(a.T);
    if constexpr (LDS_TOTALS) {
        for (uint32_t t = threadIdx.x; t < T; t += kDeltaThreads) lds_totals[t] = 0;
        __syncthreads();
    }
    const unsigned long long stride = static_cast<unsigned long long>(gridDim.x) * kDeltaThreads;
    const unsigned long long first = static_cast<unsigned long long>(blockIdx.x) * kDeltaThreads + threadIdx.x;

    // 128-bit region: groups of 4 consecutive cells, kDeltaVpt groups per lane
    // and step, kDeltaThreads groups apart.  The counts are loaded together with the
    // deltas (not after their sum is known), so that the latencies overlap; a
    // group whose summed delta is zero is not written back.
    const unsigned long long groups = a.n_vec / 4;
    u32x4 *counts4 = reinterpret_cast<u32x4 *>(a.counts);
    for (unsigned long long g0 = first + static_cast<unsigned long long>(blockIdx.x) * kDeltaThreads * (kDeltaVpt - 1);
         g0 < groups; g0 += stride * kDeltaVpt) {
        u32x4 sum[kDeltaVpt], old[kDeltaVpt];
        bool on[kDeltaVpt];
#pragma unroll
        for (int v = 0; v < kDeltaVpt; ++v) {
            const unsigned long long g = g0 + static_cast<unsigned long long>(v) * kDeltaThreads;
            on[v] = g < groups;
            sum[v] = u32x4{0, 0, 0, 0};
            old[v] = on[v] ? counts4[g] : u32x4{0, 0, 0, 0};
        }
        for (int k0 = 0; k0 < a.K; k0 += kDeltaChunk) {
            u32x4 x[kDeltaChunk][kDeltaVpt];
#pragma unroll
            for (int c = 0; c < kDeltaChunk; ++c) {
#pragma unroll
                for (int v = 0; v < kDeltaVpt; ++v) {
                    x[c][v] = u32x4{0, 0, 0, 0};
                    if (k0 + c < a.K && on[v]) {
                        x[c][v] = __builtin_nontemporal_load(
                            reinterpret_cast<const u32x4 *>(a.delta[k0 + c]) + g0 +
                            static_cast<unsigned long long>(v) * kDeltaThreads);
                    }
                }
            }
#pragma unroll
            for (int c = 0; c < kDeltaChunk; ++c) {
#pragma unroll
                for (int v = 0; v < kDeltaVpt; ++v) sum[v] += x[c][v];
            }
        }
#pragma unroll
        for (int v = 0; v < kDeltaVpt; ++v) {
            if (on[v] && (sum[v].x | sum[v].y | sum[v].z | sum[v].w) != 0) {
                const unsigned long long g = g0 + static_cast<unsigned long long>(v) * kDeltaThreads;
                counts4[g] = old[v] + sum[v];
                uint32_t col = static_cast<uint32_t>((g * 4) % T);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    add_to_total<LDS_TOTALS>(a, lds_totals, col, sum[v][j]);
                    col = col + 1 == T ? 0 : col + 1;
                }
            }
        }
    }
    // Cell-wise region: the ragged tail, or everything when a pointer is not
    // 16-byte aligned.
    const unsigned long long left = a.n_cells - a.n_vec;
    for (unsigned long long i = first; i < left; i += stride) {
        const unsigned long long cell = a.n_vec + i;
        uint32_t sum = 0;
        for (int k = 0; k < a.K; ++k) sum += static_cast<uint32_t>(__builtin_nontemporal_load(a.delta[k] + cell));
        if (sum != 0) {
            a.counts[cell] = static_cast<int32_t>(static_cast<uint32_t>(a.counts[cell]) + sum);
            add_to_total<LDS_TOTALS>(a, lds_totals, static_cast<uint32_t>(cell % T), sum);
        }
    }
    if constexpr (LDS_TOTALS) {
        __syncthreads();
        if (a.totals != nullptr) {
            for (uint32_t t = threadIdx.x; t < T; t += kDeltaThreads) {
                const int32_t v = lds_totals[t];
                if (v != 0) add_relaxed(a.totals + t, v);
            }
        }
    }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------

size_t align_up(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// Upper bounds of the work lists the plan kernel builds on the device: the sum
// over ranges of ceil(n_r / step) is at most n / step + number of ranges.
// Words cleared before every call: histogram, padded cursors, the format flag.
size_t zeroed_words(uint32_t n_tiles, uint32_t n_coarse)
{
    return n_tiles + static_cast<size_t>(kCursorStride) * (kMaxCoarse + n_tiles) + 1;
}

size_t max_fine_steps(long long n, uint32_t n_coarse) { return static_cast<size_t>(n / kPartTile) + n_coarse; }
size_t max_acc_items(long long n, uint32_t n_tiles) { return static_cast<size_t>(n / kAccChunk) + n_tiles; }

// Whether the binned path can serve this shape, and its scratch layout.
// Returns the scratch size in bytes (0 when the shape is not eligible).
size_t plan_layout(int32_t V, int32_t T, long long n, char *ws, BinPlan *plan)
{
    if (V < 1 || T < 1 || n < 1 || n > 0x7fffffffll) return 0;
    const unsigned long long cells = static_cast<unsigned long long>(V) * static_cast<unsigned long long>(T);
    const unsigned long long tiles = (cells + kTileCells - 1) >> kTileBits;
    if (tiles > kMaxTiles) return 0;
    const uint32_t n_tiles = static_cast<uint32_t>(tiles);
    if (n < kMinBinnedTriples + kMinBinnedTriplesPerTile * n_tiles) return 0;
    const uint32_t n_coarse = (n_tiles + kFinePerCoarse - 1) >> kFineBits;
    if (n_coarse > kMaxCoarse) return 0;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = ws != nullptr ? ws + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    // hist, coarse_cursor, fine_cursor are contiguous: cleared by one kernel.
    const size_t n_zeroed = zeroed_words(n_tiles, n_coarse);
    char *hist = take(sizeof(uint32_t) * n_zeroed);
    char *tile_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *coarse_part_start = take(sizeof(uint32_t) * (n_coarse + 1));
    char *chunk_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *hot_chunk_start = take(sizeof(uint32_t) * (kMaxCoarse + 1));
    char *hot_tile = take(sizeof(uint32_t) * kMaxCoarse);
    char *tmp_start = take(sizeof(uint32_t) * (n_coarse + 1));
    char *digit_start = take(sizeof(uint32_t) * kMaxCoarse);
    char *hot_bits = take(sizeof(uint32_t) * (kHotWords + 1));
    char *hot_before = take(sizeof(uint32_t) * (kHotWords + 1));
    char *tmp = take(sizeof(Record) * static_cast<size_t>(n));
    char *sorted = take(sizeof(Record) * static_cast<size_t>(n));
    if (plan != nullptr) {
        plan->hist = reinterpret_cast<uint32_t *>(hist);
        plan->coarse_cursor = plan->hist + n_tiles;
        plan->fine_cursor = plan->coarse_cursor + static_cast<size_t>(kCursorStride) * kMaxCoarse;
        plan->wide_flag = plan->fine_cursor + static_cast<size_t>(kCursorStride) * n_tiles;
        plan->tile_start = reinterpret_cast<uint32_t *>(tile_start);
        plan->coarse_part_start = reinterpret_cast<uint32_t *>(coarse_part_start);
        plan->chunk_start = reinterpret_cast<uint32_t *>(chunk_start);
        plan->hot_chunk_start = reinterpret_cast<uint32_t *>(hot_chunk_start);
        plan->hot_tile = reinterpret_cast<uint32_t *>(hot_tile);
        plan->tmp_start = reinterpret_cast<uint32_t *>(tmp_start);
        plan->digit_start = reinterpret_cast<uint32_t *>(digit_start);
        plan->hot_bits = reinterpret_cast<uint32_t *>(hot_bits);
        plan->hot_before = reinterpret_cast<uint32_t *>(hot_before);
        plan->tmp = tmp;
        plan->sorted = sorted;
        plan->n_tiles = n_tiles;
        plan->n_coarse = n_coarse;
        plan->n_cells = cells;
    }
    return off;
}

bool launched() { return hipGetLastError() == hipSuccess; }

}  // namespace

extern "C" size_t mlf_sparse_workspace_bytes(int32_t V, int32_t T, int64_t total_triples)
{
    return plan_layout(V, T, total_triples, nullptr, nullptr);
}

extern "C" mlf_status mlf_sparse_scatter_add(int32_t *counts, int32_t *totals, int32_t V,
                                             int32_t T, const int32_t *const *triple_ptrs,
                                             const int64_t *n_triples, int K, void *workspace,
                                             size_t workspace_bytes, int32_t *n_rejected,
                                             mlf_stream stream)
{
    if (counts == nullptr || V < 1 || T < 1 || K < 0) return MLF_EINVAL;
    if (K > MLF_MAX_K) return MLF_EUNSUPPORTED;
    if (K > 0 && (triple_ptrs == nullptr || n_triples == nullptr)) return MLF_EINVAL;

    SparseArgs a;
    long long longest = 0, total = 0;
    int used = 0;
    for (int k = 0; k < K; ++k) {
        if (n_triples[k] < 0) return MLF_EINVAL;
        if (n_triples[k] == 0) continue;
        if (triple_ptrs[k] == nullptr) return MLF_EINVAL;
        if (reinterpret_cast<uintptr_t>(triple_ptrs[k]) % 4 != 0) return MLF_EALIGN;
        if (reinterpret_cast<uintptr_t>(counts) % 4 != 0) return MLF_EALIGN;
        a.triples[used] = triple_ptrs[k];
        a.n_triples[used] = n_triples[k];
        if (n_triples[k] > longest) longest = n_triples[k];
        total += n_triples[k];
        ++used;
    }
    if (used == 0) return MLF_OK;
    for (int k = used; k < MLF_MAX_K; ++k) {
        a.triples[k] = nullptr;
        a.n_triples[k] = 0;
    }
    a.counts = counts;
    a.totals = totals;
    a.rejected = n_rejected;
    a.V = V;
    a.T = T;
    hipStream_t s = static_cast<hipStream_t>(stream);

    // The first pass over the triples: enough workgroups to fill the chip, few
    // enough that their merges of private totals / histograms stay small next to
    // the streamed triples.
    long long per_buffer = (longest + kScanBlock * 16 - 1) / (kScanBlock * 16);
    const long long cap = (kScanWorkgroups + used - 1) / used;
    if (per_buffer > cap) per_buffer = cap;
    if (per_buffer < 1) per_buffer = 1;
    const dim3 scan_grid(static_cast<unsigned>(per_buffer), static_cast<unsigned>(used));
    bool lds_totals = totals != nullptr && T <= kMaxLdsTopics;
    size_t totals_lds = lds_totals ? static_cast<size_t>(T) * sizeof(int32_t) : 0;

    BinPlan plan = {};
    const size_t need = plan_layout(V, T, total, static_cast<char *>(workspace), &plan);
    const bool binned = need != 0 && workspace != nullptr && workspace_bytes >= need &&
                        reinterpret_cast<uintptr_t>(workspace) % 256 == 0;
    if (!binned) {
        if (lds_totals) {
            scan_triples_kernel<false, true><<<scan_grid, dim3(kScanBlock), totals_lds, s>>>(a, plan);
        } else {
            scan_triples_kernel<false, false><<<scan_grid, dim3(kScanBlock), 0, s>>>(a, plan);
        }
        return launched() ? MLF_OK : MLF_EHIP;
    }

    // 1. clear the counters, 2. histogram (+ totals, rejects), 3. offsets,
    // 4. coarse partition, 5. fine partition, 6. accumulate and merge.
    const uint32_t n_clear = static_cast<uint32_t>(zeroed_words(plan.n_tiles, plan.n_coarse));
    clear_kernel<<<dim3((n_clear + kThreads - 1) / kThreads), dim3(kThreads), 0, s>>>(plan.hist, n_clear);
    if (!launched()) return MLF_EHIP;
    const size_t hist_lds = static_cast<size_t>(plan.n_tiles) * sizeof(uint32_t);
    if (totals_lds + hist_lds <= 65536) {
        if (lds_totals) {
            scan_triples_kernel<true, true><<<scan_grid, dim3(kScanBlock), totals_lds + hist_lds, s>>>(a, plan);
        } else {
            scan_triples_kernel<true, false><<<scan_grid, dim3(kScanBlock), hist_lds, s>>>(a, plan);
        }
    } else if (lds_totals && T <= kBigTopics) {
        // More than 64 KiB of histogram and totals: the variant with a static array.
        scan_triples_kernel<true, true, true><<<scan_grid, dim3(kScanBlock), 0, s>>>(a, plan);
    } else {
        scan_triples_kernel<true, false, true><<<scan_grid, dim3(kScanBlock), 0, s>>>(a, plan);
    }
    if (!launched()) return MLF_EHIP;
    plan_kernel<<<dim3(1), dim3(kPlanThreads), 0, s>>>(plan);
    if (!launched()) return MLF_EHIP;
    const unsigned steps_per_buffer = static_cast<unsigned>((longest + kPartTile - 1) / kPartTile);
    coarse_partition_kernel<<<dim3(steps_per_buffer, static_cast<unsigned>(used)), dim3(kPartThreads), 0, s>>>(a, plan);
    if (!launched()) return MLF_EHIP;
    const unsigned fine_steps = static_cast<unsigned>(max_fine_steps(total, plan.n_coarse));
    fine_partition_kernel<<<dim3(fine_steps), dim3(kPartThreads), 0, s>>>(plan);
    if (!launched()) return MLF_EHIP;
    const unsigned acc_items = static_cast<unsigned>(max_acc_items(total, plan.n_tiles));
    accumulate_kernel<<<dim3(acc_items), dim3(kAccThreads), 0, s>>>(counts, plan);
    return launched() ? MLF_OK : MLF_EHIP;
}

extern "C" mlf_status mlf_counts_add_dense(int32_t *counts, int32_t *totals, int32_t V, int32_t T,
                                           const int32_t *const *delta_ptrs, int K,
                                           mlf_stream stream)
{
    if (counts == nullptr || V < 1 || T < 1 || K < 0) return MLF_EINVAL;
    if (K > MLF_MAX_K) return MLF_EUNSUPPORTED;
    if (K == 0) return MLF_OK;
    if (delta_ptrs == nullptr) return MLF_EINVAL;
    if (reinterpret_cast<uintptr_t>(counts) % 4 != 0) return MLF_EALIGN;
    DeltaArgs a;
    a.n_cells = static_cast<unsigned long long>(V) * static_cast<unsigned long long>(T);
    const uintptr_t bytes = static_cast<uintptr_t>(a.n_cells) * 4;
    const uintptr_t c_lo = reinterpret_cast<uintptr_t>(counts);
    bool aligned16 = c_lo % 16 == 0;
    for (int k = 0; k < K; ++k) {
        const uintptr_t d_lo = reinterpret_cast<uintptr_t>(delta_ptrs[k]);
        if (d_lo == 0) return MLF_EINVAL;
        if (d_lo % 4 != 0) return MLF_EALIGN;
        if (d_lo < c_lo + bytes && c_lo < d_lo + bytes) return MLF_EINVAL;     // overlaps counts
        aligned16 = aligned16 && d_lo % 16 == 0;
        a.delta[k] = delta_ptrs[k];
    }
    for (int k = K; k < MLF_MAX_K; ++k) a.delta[k] = nullptr;
    a.counts = counts;
    a.totals = totals;
    a.n_vec = aligned16 ? a.n_cells / 4 * 4 : 0;
    a.K = K;
    a.T = T;
    const unsigned long long work = a.n_vec / 4 > a.n_cells - a.n_vec ? a.n_vec / 4 : a.n_cells - a.n_vec;
    unsigned long long tiles = (work + kDeltaThreads * kDeltaVpt - 1) / (kDeltaThreads * kDeltaVpt);
    if (tiles > kDeltaMaxGrid) tiles = kDeltaMaxGrid;
    if (tiles < 1) tiles = 1;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (totals != nullptr && T <= kMaxLdsTopics) {
        dense_delta_kernel<true><<<dim3(static_cast<unsigned>(tiles)), dim3(kDeltaThreads),
                                   static_cast<size_t>(T) * sizeof(int32_t), s>>>(a);
    } else {
        dense_delta_kernel<false><<<dim3(static_cast<unsigned>(tiles)), dim3(kDeltaThreads), 0, s>>>(a);
    }
    return launched() ? MLF_OK : MLF_EHIP;
}
