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
// Binned path (needs scratch).  The triples cross HBM once.  They are grouped
// by the 128 KiB tile of counts[] they fall into (a two-level partition: 128
// fine tiles per coarse range, so that every partition step writes contiguous
// runs; the heaviest tiles get a digit of their own at the coarse level and skip
// the fine one).  Where the groups go is planned from a SAMPLE of the triples
// (every 64th block of 256, or denser for matrices of many tiles): every tile
// gets room for its estimated share plus five standard deviations.  A record
// that finds its group full is added to counts[] with a global atomic on the
// spot instead, so the result does not depend on how good the estimate was;
// only the speed does (a batch whose sample says nothing about the rest
// degrades to the direct path's cost).  One workgroup then owns a tile at a
// time: it accumulates the tile's records with LDS atomics into a private
// 32768-cell image and merges the image into counts[] with contiguous 128-bit
// read-modify-writes (or contiguous atomics when a heavy tile is shared by
// several workgroups).  Global atomic traffic drops from one operation per
// triple to one per touched cache line per workgroup, and everything else is
// streaming.
//
// In both paths the T-entry totals vector, which every triple hits, is kept in
// LDS per workgroup and merged into totals[] once at the end.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "launch.h"
#include "mlfabric.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxLdsTopics = 16384;     // direct path: totals privatised in LDS up to 64 KiB

// ---- geometry of the binned path (frozen results of sweeps on MI355X) ---------
constexpr int kTileBits = 15;                    // log2 of the cells per LDS image (128 KiB)
constexpr uint32_t kTileCells = 1u << kTileBits;
constexpr int kFineBits = 7;                     // log2 of the fine tiles per coarse range
constexpr uint32_t kFinePerCoarse = 1u << kFineBits;
constexpr uint32_t kMaxCoarse = 256;             // digits of the coarse level (one counter per lane)
constexpr uint32_t kMaxTiles = 32768;            // tiles a call may span (LDS histogram, plan tables)
constexpr int kPartThreads = 1024;               // lanes of a partition workgroup
constexpr int kPartItems = 8;                    // records per lane in a partition step
constexpr uint32_t kPartTile = kPartThreads * kPartItems;      // records per step
constexpr unsigned kCoarseWorkgroups = 512;      // persistent workgroups of the coarse level (2 per CU)
constexpr int kCoarseLdsTopics = 8192;           // coarse level: totals privatised in LDS up to 32 KiB
// Output cursors sit this many words apart: every partition step of a range
// bumps the same cursors, and atomics on one cache line are served one by one.
constexpr uint32_t kCursorStride = 32;
constexpr int kAccThreads = 1024;                // lanes of an accumulate workgroup
constexpr uint32_t kAccChunk = 1u << 18;         // records per accumulate work item
constexpr int kScanBlock = 1024;                 // lanes of a direct-path / sample workgroup
constexpr int kScanWorkgroups = 512;             // direct-path workgroups of a call, about
constexpr int kScanUnroll = 2;                   // triples per lane and step of the direct path
constexpr int kPlanThreads = 1024;               // lanes of the one plan workgroup
// The sample: blocks of kSampleBlock consecutive triples, every `period`-th
// block of each buffer; period = n / (kSamplePerTile * tiles), i.e. about
// kSamplePerTile sampled triples per tile, at most kSampleMaxPeriod and at
// least 1 (then the "sample" is every triple and the plan is exact).
constexpr long long kSampleBlock = 256;
constexpr long long kSampleMaxPeriod = 64;
constexpr long long kSamplePerTile = 256;
constexpr unsigned kSampleWorkgroups = 128;
// Room per tile: (h + kRoomSigmas * sqrt(h) + kRoomFloor) * (triples per sampled
// triple), h = the tile's count in the sample.
constexpr float kRoomSigmas = 5.0f;
constexpr float kRoomFloor = 8.0f;
// The binned path has a fixed cost (six launches, one accumulate workgroup per
// non-empty tile); the direct path is cheaper below about this many triples
// (measured crossovers: 0.25 M triples on a 31-tile matrix, 2 M on 3,052 tiles).
constexpr long long kMinBinnedTriples = 1 << 18;
constexpr long long kMinBinnedTriplesPerTile = 600;

struct SparseArgs {
    const int32_t *triples[MLF_MAX_K];
    long long n_triples[MLF_MAX_K];
    uint32_t step_start[MLF_MAX_K + 1];  // coarse partition steps in the buffers before each one
    uint32_t sample_start[MLF_MAX_K + 1];// sampled blocks in the buffers before each one
    int32_t *counts;
    int32_t *totals;
    int32_t *rejected;
    int V;
    int T;
    int n_buffers;                       // buffers that hold triples
    int sample_period;                   // every sample_period-th block of kSampleBlock triples is sampled
};

// Records travel through the scratch as ONE word, the same at every stage: the
// low kCoarseShift bits are the cell index inside the record's coarse range (the
// range itself is implied by where the record lies: its group in `tmp`, its
// tile in `sorted`), the bits above are the delta.  The low kTileBits bits are the
// cell inside the tile, which is all the accumulate step needs.  LDA deltas are
// almost always +-1.  A delta outside [-kSmallDeltaLimit, kSmallDeltaLimit)
// never becomes a record: the coarse level adds it to counts[] with a global
// atomic instead, which costs what the direct path costs for that triple.  A
// zero delta changes nothing and is dropped, so a record word is never 0.
constexpr int kCoarseShift = kTileBits + kFineBits;
constexpr uint32_t kRangeMask = (1u << kCoarseShift) - 1;
constexpr int32_t kSmallDeltaLimit = 1 << (31 - kCoarseShift);

__device__ __forceinline__ uint32_t pack_record(uint32_t cell, int32_t delta)
{
    return (cell & kRangeMask) | (static_cast<uint32_t>(delta) << kCoarseShift);
}

__device__ __forceinline__ int32_t record_delta(uint32_t v) { return static_cast<int32_t>(v) >> kCoarseShift; }

// Control block of the binned path, carved out of the caller's scratch.  All
// the "start" tables describe ROOM (planned from the sample); how many records
// actually arrived in a group is the smaller of its cursor and its room.
struct BinPlan {
    uint32_t *hist;               // [n_tiles]   sampled triples per tile    (zeroed)
    uint32_t *coarse_cursor;      // [kMaxCoarse * kCursorStride] records that asked for a place per
                                  //                             digit of the coarse level (zeroed)
    uint32_t *fine_cursor;        // [n_tiles * kCursorStride]  the same per tile, fine level (zeroed)
    uint32_t *tile_start;         // [n_tiles+1] where each tile's room begins in `sorted`
    uint32_t *coarse_part_start;  // [n_coarse+1] fine partition steps before each coarse range
    uint32_t *chunk_start;        // [n_tiles+1] accumulate work items of the tiles that are not hot,
                                  //             before each tile
    uint32_t *hot_chunk_start;    // [kMaxCoarse+1] accumulate work items before each hot tile; the hot
                                  //             tiles' items come first in the launch
    uint32_t *hot_tile;           // [kMaxCoarse] tile of each hot digit
    uint32_t *tmp_start;          // [n_coarse+1] where each coarse range's room begins in `tmp`
    uint32_t *digit_start;        // [kMaxCoarse] first output index of each digit of the coarse level,
                                  //              counted from tmp[0]: in tmp for a coarse range, in
                                  //              sorted (sorted_base + ...) for a hot tile
    uint32_t *digit_room;         // [kMaxCoarse] room of each digit of the coarse level
    uint8_t *tile_digit;          // [n_tiles] digit of each tile at the coarse level: its coarse range,
                                  //              or n_coarse + its rank among the hot tiles
    uint32_t *tmp;                // [n_slots] records grouped by coarse range
    uint32_t *sorted;             // [n_slots] records grouped by tile; sorted = tmp + sorted_base
    uint32_t sorted_base;
    uint32_t n_tiles;
    uint32_t n_coarse;
    uint32_t n_slots;             // words in tmp and in sorted
    float per_sampled;            // triples of the call per sampled triple (>= 1)
    unsigned long long n_cells;   // V * T
};

// Records of a group: what asked for a place, capped by the room.
__device__ __forceinline__ uint32_t arrived(const uint32_t *cursor, uint32_t room)
{
    return min(*cursor, room);
}

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

// Inclusive prefix sum over the 64 lanes of a wavefront with cross-lane moves of
// the vector pipeline (no LDS): shifts by 1, 2, 4 and 8 inside each row of 16
// lanes (a lane without a source adds 0), then the last lane of rows 0 and 2
// into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t v)
{
    v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);     // row_shr:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);     // row_shr:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);     // row_shr:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);     // row_shr:8
    v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false);     // row_bcast:15 into rows 1, 3
    v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false);     // row_bcast:31 into rows 2, 3
    return v;
}

// For each of the N records of every lane: counter[bin[i]] += 1 if live[i], and
// rank[i] = the value the record would have seen had the records gone one by one
// (its rank in its bin; no two live records of a bin get the same).  Skewed data
// puts many lanes of a wavefront into one bin, and LDS atomics on one address
// are served one lane at a time; so for every i the lanes that share the bin of
// the first live lane are counted with a ballot and added by that lane alone,
// and only the others add for themselves: one LDS atomic instruction per i (the
// group's other members sit it out).  The N atomics of a lane are issued back to
// back and waited for once, so that their trips through the LDS overlap: with
// two 16-wavefront workgroups on a CU a single trip takes several hundred
// cycles.  Must be called by whole wavefronts.
template <int N>
__device__ __forceinline__ void wave_rank_all(uint32_t *counter, const uint32_t (&bin)[N],
                                              const bool (&live)[N], uint32_t (&rank)[N])
{
    const int lane = static_cast<int>(threadIdx.x & 63);
    unsigned long long group[N];
    int first[N];
    bool grouped[N];
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const unsigned long long live_mask = __ballot(live[i]);
        // (with no live lane the lookups read lane 63: harmless, nobody is grouped then)
        first[i] = (__ffsll(static_cast<long long>(live_mask)) - 1) & 63;          // uniform
        grouped[i] = live[i] && bin[i] == broadcast(bin[i], first[i]);
        group[i] = __ballot(grouped[i]);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        rank[i] = 0;
        if (live[i] && (!grouped[i] || lane == first[i])) {
            rank[i] = lds_fetch_add(&counter[bin[i]],
                                    grouped[i] ? static_cast<uint32_t>(__popcll(group[i])) : 1u);
        }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
        const uint32_t base = broadcast(rank[i], first[i]);
        if (grouped[i]) rank[i] = base + lanes_below(group[i]);
    }
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

// The same for the triple that starts `offset` bytes after `base` (a wavefront-
// uniform address plus a 32-bit lane offset: one 96-bit load).
__device__ __forceinline__ bool load_triple_at(const char *base, uint32_t offset, int V, int T,
                                               int &word, int &topic, int &delta)
{
    typedef int32_t i32x3 __attribute__((ext_vector_type(3)));
    typedef i32x3 __attribute__((aligned(4))) i32x3_unaligned;
    const i32x3 v = __builtin_nontemporal_load(reinterpret_cast<const i32x3_unaligned *>(base + offset));
    word = v.x;
    topic = v.y;
    delta = v.z;
    return static_cast<unsigned>(word) < static_cast<unsigned>(V) &&
           static_cast<unsigned>(topic) < static_cast<unsigned>(T);
}

// Direct path; blockIdx.y = worker buffer, blockIdx.x = share of that buffer.
// Every valid triple is added to counts[] with a global atomic; the totals are
// kept in LDS (dynamic, T entries) when LDS_TOTALS, and the rejected triples
// are counted.
template <bool LDS_TOTALS>
__global__ __launch_bounds__(kScanBlock) void direct_kernel(const SparseArgs a)
{
    extern __shared__ int32_t lds_totals[];
    const int T = a.T;
    const bool want_totals = a.totals != nullptr;
    if constexpr (LDS_TOTALS) {
        for (int t = threadIdx.x; t < T; t += kScanBlock) lds_totals[t] = 0;
        __syncthreads();
    }
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
            add_relaxed(a.counts + (static_cast<long long>(word[u]) * T + topic[u]), delta[u]);
            if (want_totals) {
                if constexpr (LDS_TOTALS) {
                    lds_add(&lds_totals[topic[u]], delta[u]);
                } else {
                    add_relaxed(a.totals + topic[u], delta[u]);
                }
            }
        }
    }
    if constexpr (LDS_TOTALS) {
        __syncthreads();
        if (want_totals) {
            for (int t = threadIdx.x; t < T; t += kScanBlock) {
                const int32_t v = lds_totals[t];
                if (v != 0) add_relaxed(a.totals + t, v);
            }
        }
    }
    if (a.rejected != nullptr) {
        // Wavefront sum of the per-lane reject counts, one atomic per wavefront.
        for (int off = 32; off > 0; off >>= 1) n_bad += __shfl_down(n_bad, off, 64);
        if ((threadIdx.x & 63) == 0 && n_bad != 0) add_relaxed(a.rejected, n_bad);
    }
}

// The sample of the binned path: per-tile counts of the valid, record-sized
// triples in every sample_period-th block of kSampleBlock triples of every
// buffer.  The sampled blocks of all buffers form one list; a quarter of a
// workgroup takes a block, and every lane has the loads of kSampleUnroll blocks
// in flight.  The histogram is built in LDS (dynamic, n_tiles words; BIG = a
// static array for more than 16,384 tiles) and merged into plan.hist with one
// atomic per non-empty bin.
constexpr int kSampleUnroll = 4;

template <bool BIG>
__global__ __launch_bounds__(kScanBlock) void sample_kernel(const SparseArgs a, const BinPlan plan)
{
    extern __shared__ int32_t dynamic_lds[];
    __shared__ int32_t static_lds[BIG ? kMaxTiles : 1];
    uint32_t *lds_hist = reinterpret_cast<uint32_t *>(BIG ? static_lds : dynamic_lds);
    // The per-buffer tables are looked up per lane: from LDS, not from the
    // kernel-argument segment (a chain of dependent global loads otherwise).
    __shared__ uint32_t s_start[MLF_MAX_K + 1];
    __shared__ long long s_count[MLF_MAX_K];
    __shared__ const int32_t *s_triples[MLF_MAX_K];
    for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kScanBlock) lds_hist[b] = 0;
    if (threadIdx.x <= MLF_MAX_K) s_start[threadIdx.x] = a.sample_start[threadIdx.x];
    if (threadIdx.x < MLF_MAX_K) {
        s_count[threadIdx.x] = a.n_triples[threadIdx.x];
        s_triples[threadIdx.x] = a.triples[threadIdx.x];
    }
    __syncthreads();
    constexpr uint32_t kBlocksAtOnce = kScanBlock / kSampleBlock;     // sampled blocks per workgroup and load
    const uint32_t within = threadIdx.x % kSampleBlock;
    const uint32_t n_sampled = s_start[a.n_buffers];
    const uint32_t stride = gridDim.x * kBlocksAtOnce;
    for (uint32_t q0 = blockIdx.x * kBlocksAtOnce + threadIdx.x / kSampleBlock; q0 < n_sampled;
         q0 += stride * kSampleUnroll) {
        int word[kSampleUnroll], topic[kSampleUnroll], delta[kSampleUnroll];
        bool ok[kSampleUnroll];
#pragma unroll
        for (int u = 0; u < kSampleUnroll; ++u) {
            const uint32_t q = q0 + u * stride;                        // sampled block in the list
            // its buffer: the last one that starts at or before q
            int lo = 0, hi = a.n_buffers;
            while (hi - lo > 1) {
                const int mid = (lo + hi) / 2;
                if (s_start[mid] <= q) lo = mid; else hi = mid;
            }
            const long long r = static_cast<long long>(q - s_start[lo]) * a.sample_period * kSampleBlock + within;
            const long long m = s_count[lo];                           // >= 1
            const bool there = q < n_sampled && r < m;
            // (no branch around the load: a lane with nothing to sample reloads the last triple)
            ok[u] = load_triple(s_triples[lo], there ? r : m - 1, a.V, a.T, word[u], topic[u], delta[u]) && there;
        }
#pragma unroll
        for (int u = 0; u < kSampleUnroll; ++u) {
            if (ok[u] && delta[u] != 0 && delta[u] >= -kSmallDeltaLimit && delta[u] < kSmallDeltaLimit) {
                const uint32_t cell = static_cast<uint32_t>(word[u]) * static_cast<uint32_t>(a.T) +
                                      static_cast<uint32_t>(topic[u]);
                wave_count(lds_hist, cell >> kTileBits);
            }
        }
    }
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kScanBlock) {
        const uint32_t v = lds_hist[b];
        if (v != 0) fetch_add_relaxed(plan.hist + b, v);
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
// the workgroup: a scan inside each wavefront, then the wavefront totals
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
    for (int k = 0; k < N; ++k) incl[k] = wave_inclusive_sum(v[k]);
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

// One workgroup: turns the sampled tile histogram into the room every later
// step works in.
//
// Room of a tile: (h + kRoomSigmas * sqrt(h) + kRoomFloor) * per_sampled records,
// h = its count in the sample; the running total is cut off at n_slots, the size
// of the arrays, so that whatever the sample says no index leaves them.
//
// Heavy tiles skip the fine level.  The coarse level has kMaxCoarse digits and
// needs n_coarse of them for the coarse ranges; each spare digit is given to one
// of the heaviest tiles ("hot"), whose records the coarse level then writes
// straight to their final place in `sorted`.  Under a Zipf law a few hundred
// tiles hold most of the records, so most records are moved once instead of
// twice.  The hot tiles are those with at least `threshold` sampled triples,
// the smallest power-of-two fraction of the sample that leaves no more hot tiles
// than spare digits.  The digit of every tile (its coarse range, or n_coarse +
// its rank among the hot tiles) is published as a table of one byte per tile.
//
// Lane i looks after `per_lane` CONSECUTIVE tiles, so every table over the
// tiles takes a serial pass inside each lane plus one block scan of the lane
// sums; the per-tile rooms are kept in LDS between the passes and the sampled
// counts are read again in each (they stay cached).
constexpr int kHotShifts = 24;      // a hot tile holds at least total >> (kHotShifts - 1) sampled triples
constexpr uint32_t kWantSplit = 20; // lane sums of rooms are scanned as two words of 20 and 12 bits

__global__ __launch_bounds__(kPlanThreads) void plan_kernel(const BinPlan plan)
{
    static_assert(kMaxCoarse <= kPlanThreads, "the tables over coarse digits take one round");
    static_assert(kMaxTiles / kPlanThreads <= 32, "a lane's hot tiles are one bit each of a word");
    __shared__ uint32_t wave_sums[3][kPlanWaves];
    __shared__ uint32_t tiles_at_least[kHotShifts];
    __shared__ uint32_t hot_in_range[kMaxCoarse];     // room of the hot tiles of each coarse range
    __shared__ uint32_t range_start[kMaxCoarse + 1];  // tile_start at the first tile of each coarse range
    __shared__ uint32_t hot_room[kMaxCoarse];         // room of each hot tile, by its rank
    __shared__ uint32_t s_threshold;
    __shared__ uint32_t room[kMaxTiles];              // room per tile
    const uint32_t n_tiles = plan.n_tiles;
    const uint32_t n_coarse = plan.n_coarse;
    const uint32_t n_slots = plan.n_slots;            // < 2^31
    const uint32_t lane = threadIdx.x & 63;
    const uint32_t per_lane = (n_tiles + kPlanThreads - 1) / kPlanThreads;
    const uint32_t lo = min(threadIdx.x * per_lane, n_tiles);
    const uint32_t hi = min(lo + per_lane, n_tiles);

    if (threadIdx.x < kHotShifts) tiles_at_least[threadIdx.x] = 0;
    if (threadIdx.x < kMaxCoarse) hot_in_range[threadIdx.x] = 0;

    // Pass 1: the room every tile asks for, each cut at n_slots; lane sums.
    unsigned long long asked = 0;
    uint32_t sampled = 0;
#pragma unroll 4
    for (uint32_t b = lo; b < hi; ++b) {
        const uint32_t h = plan.hist[b];
        const float hf = static_cast<float>(h);
        const float want = (hf + kRoomSigmas * sqrtf(hf) + kRoomFloor) * plan.per_sampled + 1.0f;
        const uint32_t w = static_cast<uint32_t>(fminf(want, static_cast<float>(n_slots)));
        room[b] = w;
        asked += w;
        sampled += h;
    }
    uint32_t first;                                   // tile_start of the lane's first tile
    uint32_t sample;
    {
        const uint32_t mine = asked < n_slots ? static_cast<uint32_t>(asked) : n_slots;
        const uint32_t v[3] = {mine & ((1u << kWantSplit) - 1), mine >> kWantSplit, sampled};
        uint32_t e[3], t[3];
        block_scan<3>(v, e, t, wave_sums);
        const unsigned long long before = (static_cast<unsigned long long>(e[1]) << kWantSplit) + e[0];
        const unsigned long long all = (static_cast<unsigned long long>(t[1]) << kWantSplit) + t[0];
        first = before < n_slots ? static_cast<uint32_t>(before) : n_slots;
        sample = t[2];
        if (threadIdx.x == 0) {
            const uint32_t placed = all < n_slots ? static_cast<uint32_t>(all) : n_slots;
            plan.tile_start[n_tiles] = placed;
            range_start[n_coarse] = placed;
        }
    }
    // tile_start: running sum inside the lane, saturating at n_slots (once the
    // total has reached n_slots every later room is 0).
    {
        uint32_t at = first;
        for (uint32_t b = lo; b < hi; ++b) {
            const uint32_t stop = min(at + room[b], n_slots);       // both terms are at most n_slots < 2^31
            plan.tile_start[b] = at;
            room[b] = stop - at;
            if ((b & (kFinePerCoarse - 1)) == 0) range_start[b >> kFineBits] = at;
            at = stop;
        }
    }

    // Pass 2: threshold of the hot tiles (on the sampled counts).
    {
        uint32_t at_least[kHotShifts];
#pragma unroll
        for (int j = 0; j < kHotShifts; ++j) at_least[j] = 0;
        for (uint32_t b = lo; b < hi; ++b) {
            const uint32_t h = plan.hist[b];
#pragma unroll
            for (int j = 0; j < kHotShifts; ++j) at_least[j] += (h != 0 && h >= (sample >> j)) ? 1u : 0u;
        }
#pragma unroll
        for (int j = 0; j < kHotShifts; ++j) {
            const uint32_t in_wave = wave_inclusive_sum(at_least[j]);
            if (lane == 63 && in_wave != 0) lds_fetch_add(&tiles_at_least[j], in_wave);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t spare = kMaxCoarse - n_coarse;
        uint32_t threshold = 0xffffffffu;                    // no hot tile
        for (int j = 0; j < kHotShifts; ++j) {
            if (tiles_at_least[j] <= spare && (sample >> j) >= 1) threshold = sample >> j;
        }
        s_threshold = threshold;
    }
    __syncthreads();
    const uint32_t threshold = s_threshold;

    // Pass 3: hot tiles (rank, room per coarse range), the digit of every tile,
    // and the accumulate work items (kAccChunk records of room each) of the tiles
    // that are not hot.
    uint32_t n_hot = 0;
    {
        uint32_t hot_mask = 0, my_hot = 0, my_items = 0;
        for (uint32_t b = lo; b < hi; ++b) {
            const uint32_t h = plan.hist[b];
            const bool hot = h != 0 && h >= threshold;
            hot_mask |= (hot ? 1u : 0u) << (b - lo);
            my_hot += hot ? 1u : 0u;
            my_items += hot ? 0u : (room[b] + kAccChunk - 1) / kAccChunk;
        }
        const uint32_t v[2] = {my_hot, my_items};
        uint32_t e[2], t[2];
        block_scan<2>(v, e, t, wave_sums);
        uint32_t slot = e[0], item = e[1], at = first;
        for (uint32_t b = lo; b < hi; ++b) {
            const bool hot = ((hot_mask >> (b - lo)) & 1u) != 0;
            const uint32_t mine = room[b];
            plan.chunk_start[b] = item;
            plan.tile_digit[b] = static_cast<uint8_t>(hot ? n_coarse + slot : b >> kFineBits);
            if (hot) {
                plan.hot_tile[slot] = b;
                plan.digit_start[n_coarse + slot] = plan.sorted_base + at;
                plan.digit_room[n_coarse + slot] = mine;
                hot_room[slot] = mine;
                lds_fetch_add(&hot_in_range[b >> kFineBits], mine);
                ++slot;
            } else {
                item += (mine + kAccChunk - 1) / kAccChunk;
            }
            at += mine;
        }
        n_hot = t[0];
        if (threadIdx.x == 0) plan.chunk_start[n_tiles] = t[1];
    }
    __syncthreads();

    // Per coarse range: the room of its tiles that still go through the fine
    // level, and the fine partition steps (kPartTile records each) that room
    // takes; per hot digit: the accumulate work items of its tile, which come
    // first in that launch so that the long ones start early.
    {
        const uint32_t c = threadIdx.x;
        uint32_t cold = 0;
        if (c < n_coarse) cold = range_start[c + 1] - range_start[c] - hot_in_range[c];
        uint32_t hot_items = 0;
        if (c < n_hot) hot_items = (hot_room[c] + kAccChunk - 1) / kAccChunk;
        const uint32_t v[3] = {cold, (cold + kPartTile - 1) / kPartTile, hot_items};
        uint32_t e[3], t[3];
        block_scan<3>(v, e, t, wave_sums);
        if (c < n_coarse) {
            plan.tmp_start[c] = e[0];          // the cold rooms add up to at most n_slots
            plan.digit_start[c] = e[0];
            plan.digit_room[c] = cold;
            plan.coarse_part_start[c] = e[1];
        }
        if (c == n_coarse) {
            plan.tmp_start[c] = t[0];
            plan.coarse_part_start[c] = t[1];
        }
        if (c >= n_coarse + n_hot && c < kMaxCoarse) {
            plan.digit_start[c] = 0;           // digits nobody uses
            plan.digit_room[c] = 0;
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

// One partition step of a workgroup: up to kPartTile record words held in
// registers are grouped by digit (< kMaxCoarse) in LDS and written out so that
// the records of one digit form one contiguous run at the place reserved for
// them.
//   word[i], live[i]    the lane's record words and whether each exists
//   dig[i]              digit of each record (0 where there is none)
//   out                 the output array
//   reserve(d, n)       asks for room for this step's n records of digit d and
//                       returns how many records of d asked before (one global
//                       atomic); called by lane 64 + d
//   room_of(d)          x = index in `out` where the room of digit d begins,
//                       y = its size; called by lane 64 + d
//   spill(d, w)         takes a record of digit d that found its group full
// The phases: (1) every record gets its rank within its digit from the LDS
// counters; (2) one wavefront scans the 256 counts, which gives every digit its
// first staging slot, while lane 64 + d issues the reservation for digit d;
// (3) the records are staged in digit order, each with its digit and rank -
// the reservations are still in flight meanwhile, and their lanes store the
// results when they arrive; (4) the stage is written out in order: a record's
// output index is its digit's reserved index plus its rank, so that a wavefront
// writes a few contiguous runs.  Must be entered by the whole workgroup, with
// s.count[] zero; leaves s.count[] zero again.
struct Staged {
    uint32_t word;
    uint32_t digit_rank;         // digit << 16 | rank within the digit in this step
};
static_assert(kPartTile <= 65536, "a rank takes 16 bits of a staged record");

struct PartitionLds {
    Staged stage[kPartTile];
    __attribute__((aligned(16))) uint32_t count[kMaxCoarse];
    uint32_t first_slot[kMaxCoarse];   // per digit: first staging slot of this step's records
    uint2 reserved[kMaxCoarse];        // per digit: x = output index of this step's first record,
                                       // y = how many of this step's records still fit there
    uint2 limit[kMaxCoarse];           // coarse level, per digit: x = first output index of its room, y = its room
    uint32_t total;
};

constexpr int kRankBatch = 4;     // records of a lane ranked together (their LDS atomics in flight at once)

template <typename Reserve, typename RoomOf, typename Spill>
__device__ __forceinline__ void partition_step(PartitionLds &s, uint32_t *__restrict__ out,
                                               const uint32_t (&word)[kPartItems],
                                               const bool (&live)[kPartItems],
                                               const uint32_t (&dig)[kPartItems], Reserve reserve,
                                               RoomOf room_of, Spill spill)
{
    static_assert(kMaxCoarse == 256 && kPartThreads >= 64 + kMaxCoarse, "one wavefront scans 4 digits per lane");
    uint32_t rank[kPartItems];
#pragma unroll
    for (int i0 = 0; i0 < kPartItems; i0 += kRankBatch) {
        uint32_t b[kRankBatch], r[kRankBatch];
        bool l[kRankBatch];
#pragma unroll
        for (int j = 0; j < kRankBatch; ++j) {
            b[j] = dig[i0 + j];
            l[j] = live[i0 + j];
        }
        wave_rank_all<kRankBatch>(s.count, b, l, r);
#pragma unroll
        for (int j = 0; j < kRankBatch; ++j) rank[i0 + j] = r[j];
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        // Exclusive scan of the 256 digit counts by one wavefront: 4 per lane
        // (one 128-bit read), then a scan of the lane sums.
        const uint32_t lane = threadIdx.x;
        const uint4 c = reinterpret_cast<const uint4 *>(s.count)[lane];
        const uint32_t sum = c.x + c.y + c.z + c.w;
        const uint32_t incl = wave_inclusive_sum(sum);
        const uint32_t run = incl - sum;
        reinterpret_cast<uint4 *>(s.first_slot)[lane] = make_uint4(run, run + c.x, run + c.x + c.y, run + c.x + c.y + c.z);
        if (lane == 63) s.total = incl;
    }
    const bool reserver = threadIdx.x >= 64 && threadIdx.x < 64 + kMaxCoarse;
    const uint32_t my_digit = (threadIdx.x - 64) & (kMaxCoarse - 1);
    uint32_t mine = 0, before = 0;
    if (reserver) {
        mine = s.count[my_digit];
        if (mine != 0) before = reserve(my_digit, mine);       // not waited for yet
    }
    __syncthreads();
    if (threadIdx.x < kMaxCoarse) s.count[threadIdx.x] = 0;     // for the next step
    uint32_t slot[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) slot[i] = s.first_slot[dig[i]];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        if (live[i]) s.stage[slot[i] + rank[i]] = Staged{word[i], (dig[i] << 16) | rank[i]};
    }
    if (mine != 0) {
        const uint2 room = room_of(my_digit);
        s.reserved[my_digit] = make_uint2(room.x + before, before < room.y ? room.y - before : 0u);
    }
    __syncthreads();
    // Write-out: every staged record of the lane is read before the first is
    // stored.  (Slots from `total` on hold leftovers of earlier steps: read,
    // since that is cheaper than a branch, and not used.)
    const uint32_t total = s.total;
    Staged e[kPartItems];
#pragma unroll
    for (int u = 0; u < kPartItems; ++u) e[u] = s.stage[u * kPartThreads + threadIdx.x];
    uint2 where[kPartItems];
#pragma unroll
    for (int u = 0; u < kPartItems; ++u) where[u] = s.reserved[(e[u].digit_rank >> 16) & (kMaxCoarse - 1)];
#pragma unroll
    for (int u = 0; u < kPartItems; ++u) {
        if (u * kPartThreads + threadIdx.x < total) {
            const uint32_t r = e[u].digit_rank & 0xffffu;
            if (r < where[u].y) {
                out[where[u].x + r] = e[u].word;
            } else {
                spill(e[u].digit_rank >> 16, e[u].word);
            }
        }
    }
}

// Coarse partition, the one pass over the triples.  A persistent grid: the
// workgroups take the steps (kPartTile triples of one buffer each) in turn and
// keep the per-topic totals in LDS over all their steps.  Valid triples become
// records: those of hot tiles go to their final place in plan.sorted, the others
// to plan.tmp, grouped by coarse range (one output index space: sorted lies
// plan.sorted_base words after tmp).  A record whose group is full, and a
// triple whose delta is too large for a record, is added to counts[] at once.
// Dynamic LDS: [digit of every tile, one byte each, padded to a word][T totals
// if LDS_TOTALS].
//
// Two workgroups share a CU (the grid is two per CU): while one waits for its
// triples or for a barrier the other works.  That takes 8 wavefronts per SIMD,
// i.e. at most 64 vector registers.
template <bool LDS_TOTALS>
__global__ __launch_bounds__(kPartThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
void coarse_partition_kernel(const SparseArgs a, const BinPlan plan)
{
    extern __shared__ uint32_t coarse_lds[];
    __shared__ PartitionLds s;
    const uint32_t digit_words = (plan.n_tiles + 3) / 4;
    const uint8_t *tile_digit = reinterpret_cast<const uint8_t *>(coarse_lds);
    int32_t *lds_totals = reinterpret_cast<int32_t *>(coarse_lds + digit_words);
    const int T = a.T;
    const bool want_totals = a.totals != nullptr;
    // (the table's allocation is padded to whole words)
    for (uint32_t w = threadIdx.x; w < digit_words; w += kPartThreads) {
        coarse_lds[w] = reinterpret_cast<const uint32_t *>(plan.tile_digit)[w];
    }
    if (threadIdx.x < kMaxCoarse) {
        s.count[threadIdx.x] = 0;
        s.limit[threadIdx.x] = make_uint2(plan.digit_start[threadIdx.x], plan.digit_room[threadIdx.x]);
    }
    if constexpr (LDS_TOTALS) {
        for (int t = threadIdx.x; t < T; t += kPartThreads) lds_totals[t] = 0;
    }
    __syncthreads();

    const uint32_t n_coarse = plan.n_coarse;
    int32_t *counts = a.counts;
    const uint32_t n_steps = a.step_start[a.n_buffers];
    const uint32_t lane_offset = threadIdx.x * 12u;         // of the lane's first triple in a step
    uint32_t n_bad = 0;                                     // of the wavefront (uniform)
    int k = 0;                                              // buffer of the current step (uniform)
#pragma unroll 1
    for (uint32_t step = blockIdx.x; step < n_steps; step += gridDim.x) {
        while (step >= a.step_start[k + 1]) ++k;            // steps only grow; k < n_buffers
        const long long base = static_cast<long long>(step - a.step_start[k]) * kPartTile;
        const long long left = a.n_triples[k] - base;       // >= 1
        const uint32_t here = left < static_cast<long long>(kPartTile) ? static_cast<uint32_t>(left) : kPartTile;
        const uint32_t last_offset = (here - 1) * 12u;
        const char *from = reinterpret_cast<const char *>(a.triples[k] + 3 * base);     // uniform
        // All of the lane's triples are loaded before the first is used.  (A
        // lane past the end reloads the step's last triple: no branch around the
        // load, so the loads of a lane issue back to back.)
        int w[kPartItems], t[kPartItems], d[kPartItems];
        bool in_range[kPartItems];
#pragma unroll
        for (int i = 0; i < kPartItems; ++i) {
            const uint32_t offset = lane_offset + static_cast<uint32_t>(i) * kPartThreads * 12u;
            in_range[i] = load_triple_at(from, min(offset, last_offset), a.V, T, w[i], t[i], d[i]);
        }
        uint32_t word[kPartItems], dig[kPartItems];
        bool live[kPartItems];
#pragma unroll
        for (int i = 0; i < kPartItems; ++i) {
            const bool there = lane_offset + static_cast<uint32_t>(i) * kPartThreads * 12u <= last_offset;
            const bool valid = there && in_range[i];
            n_bad += static_cast<uint32_t>(__popcll(__ballot(there && !in_range[i])));
            const uint32_t cell = static_cast<uint32_t>(w[i]) * static_cast<uint32_t>(T) + static_cast<uint32_t>(t[i]);
            const bool small = static_cast<uint32_t>(d[i] + kSmallDeltaLimit) < 2u * kSmallDeltaLimit;
            live[i] = valid && small && d[i] != 0;
            if (valid && !small) add_relaxed(counts + cell, d[i]);
            if (valid && want_totals && d[i] != 0) {
                if constexpr (LDS_TOTALS) {
                    lds_add(&lds_totals[t[i]], d[i]);
                } else {
                    add_relaxed(a.totals + t[i], d[i]);
                }
            }
            word[i] = pack_record(cell, d[i]);
            dig[i] = live[i] ? tile_digit[cell >> kTileBits] : 0u;
        }
        partition_step(
            s, plan.tmp, word, live, dig,
            [&](uint32_t dg, uint32_t n) { return fetch_add_relaxed(plan.coarse_cursor + dg * kCursorStride, n); },
            [&](uint32_t dg) { return s.limit[dg]; },
            [&](uint32_t dg, uint32_t v) {
                // the record's coarse range: its digit, or that of its hot tile
                const uint32_t range = dg < n_coarse ? dg : plan.hot_tile[dg - n_coarse] >> kFineBits;
                add_relaxed(counts + ((range << kCoarseShift) | (v & kRangeMask)), record_delta(v));
            });
        __syncthreads();                                    // the stage is reused by the next step
    }

    if constexpr (LDS_TOTALS) {
        __syncthreads();
        if (want_totals) {
            for (int tt = threadIdx.x; tt < T; tt += kPartThreads) {
                const int32_t v = lds_totals[tt];
                if (v != 0) add_relaxed(a.totals + tt, v);
            }
        }
    }
    // One atomic per wavefront for its rejected triples.
    if (a.rejected != nullptr && (threadIdx.x & 63) == 0 && n_bad != 0) {
        add_relaxed(a.rejected, static_cast<int32_t>(n_bad));
    }
}

// Fine partition: workgroup g takes one step of the room of one coarse range of
// plan.tmp and writes the records that arrived there to plan.sorted, grouped by
// tile (or adds them to counts[] where a tile's room is full).
__global__ __launch_bounds__(kPartThreads) void fine_partition_kernel(int32_t *counts, const BinPlan plan)
{
    __shared__ PartitionLds s;
    __shared__ uint32_t s_coarse;
    const uint32_t g = blockIdx.x;
    if (g >= plan.coarse_part_start[plan.n_coarse]) return;   // uniform
    if (threadIdx.x < 64) {
        const uint32_t c = owner_of(plan.coarse_part_start, plan.n_coarse, g);
        if (threadIdx.x == 0) s_coarse = c;
    }
    if (threadIdx.x < kMaxCoarse) s.count[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t c = s_coarse;
    const uint32_t first_tile = c << kFineBits;
    const uint32_t in_range = arrived(plan.coarse_cursor + c * kCursorStride, plan.digit_room[c]);
    const uint32_t begin = plan.tmp_start[c] + (g - plan.coarse_part_start[c]) * kPartTile;
    const uint32_t end = min(begin + kPartTile, plan.tmp_start[c] + in_range);
    if (begin >= end) return;                                 // uniform: room nobody needed
    uint32_t word[kPartItems], dig[kPartItems];
    bool live[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        const uint32_t r = begin + i * kPartThreads + threadIdx.x;
        live[i] = r < end;
        word[i] = __builtin_nontemporal_load(&plan.tmp[min(r, end - 1)]);      // (no branch around the load)
        dig[i] = live[i] ? (word[i] >> kTileBits) & (kFinePerCoarse - 1) : 0u;
    }
    partition_step(
        s, plan.sorted, word, live, dig,
        [&](uint32_t f, uint32_t n) { return fetch_add_relaxed(plan.fine_cursor + (first_tile + f) * kCursorStride, n); },
        [&](uint32_t f) {
            const uint32_t at = plan.tile_start[first_tile + f];
            return make_uint2(at, plan.tile_start[first_tile + f + 1] - at);
        },
        [&](uint32_t, uint32_t v) {
            add_relaxed(counts + ((c << kCoarseShift) | (v & kRangeMask)), record_delta(v));
        });
}

// Accumulate: workgroup g takes up to kAccChunk records of the room of one
// tile, sums those that arrived there into a private LDS image of the tile and
// merges the image into counts[].
typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
constexpr int kAccUnroll = 4;       // 128-bit record loads in flight per lane

// Adds the records [begin, end) of one tile into its LDS image.  The records
// are read with 128-bit loads (4 records each), kAccUnroll of them in flight per
// lane; the few records before the first and after the last aligned group go
// one by one.  Records are read once, here and by the fine level: their loads
// carry the no-reuse hint (-2 % on the whole call with word id = rank - 1, -8 %
// with permuted ids).  Their STORES must not: the runs a step writes start and
// end inside lines, and it is the cache that puts the pieces together (+25 %).
__device__ __forceinline__ void accumulate_records(int32_t *image, const uint32_t *__restrict__ sorted,
                                                   uint32_t begin, uint32_t end)
{
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const uint32_t first = min((begin + 3) / 4 * 4, end);
    const uint32_t last = max(first, end / 4 * 4);
    auto add_one = [&](uint32_t r) {
        const uint32_t v = __builtin_nontemporal_load(&sorted[r]);
        lds_add(&image[v & (kTileCells - 1)], record_delta(v));
    };
    if (threadIdx.x < first - begin) add_one(begin + threadIdx.x);
    if (threadIdx.x < end - last) add_one(last + threadIdx.x);

    const u32x4 *groups = reinterpret_cast<const u32x4 *>(sorted);
    const uint32_t g_end = last / 4;
    for (uint32_t g0 = first / 4 + threadIdx.x; g0 < g_end; g0 += kAccThreads * kAccUnroll) {
        u32x4 x[kAccUnroll];
#pragma unroll
        for (int u = 0; u < kAccUnroll; ++u) {
            const uint32_t g = g0 + u * kAccThreads;
            x[u] = g < g_end ? __builtin_nontemporal_load(&groups[g]) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int u = 0; u < kAccUnroll; ++u) {
            if (g0 + u * kAccThreads >= g_end) continue;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t v = x[u][j];
                lds_add(&image[v & (kTileCells - 1)], record_delta(v));
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
    // The hot tiles were filled by the coarse level (digit n_coarse + rank among
    // the hot tiles), the others by the fine level.
    const uint32_t *cursor = hot ? plan.coarse_cursor + (plan.n_coarse + s_first) * kCursorStride
                                 : plan.fine_cursor + tile * kCursorStride;
    const uint32_t in_tile = arrived(cursor, plan.tile_start[tile + 1] - plan.tile_start[tile]);
    const uint32_t begin = plan.tile_start[tile] + (g - start[s_first]) * kAccChunk;
    const uint32_t end = min(begin + kAccChunk, plan.tile_start[tile] + in_tile);
    if (begin >= end) return;                                 // uniform: room nobody needed
    accumulate_records(image, plan.sorted, begin, end);
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
        // are issued before its first store, so their latencies overlap.  A
        // 128-byte stretch (8 lanes) is written whole as soon as one of its
        // groups has changed, and counts is read and written with the no-reuse
        // hint: lines written in pieces cost the memory a read-modify-write,
        // and the matrix is far larger than any cache (both together: -13 % on
        // the whole call for 64 M LDA triples; either alone: -5 % and 0).
        u32x4 *dst4 = reinterpret_cast<u32x4 *>(dst);
        u32x4 add[kGroupsPerLane], old[kGroupsPerLane];
        bool touch[kGroupsPerLane];
#pragma unroll
        for (int k = 0; k < kGroupsPerLane; ++k) {
            const uint32_t i = k * kAccThreads + threadIdx.x;
            add[k] = __builtin_bit_cast(u32x4, image4[i]);
            const bool changed = i < groups && (add[k].x | add[k].y | add[k].z | add[k].w) != 0;
            const unsigned long long changed_lanes = __ballot(changed);
            touch[k] = i < groups && ((changed_lanes >> (threadIdx.x & 56)) & 0xffull) != 0;
            old[k] = touch[k] ? __builtin_nontemporal_load(&dst4[i]) : u32x4{0, 0, 0, 0};
        }
#pragma unroll
        for (int k = 0; k < kGroupsPerLane; ++k) {
            if (touch[k]) __builtin_nontemporal_store(old[k] + add[k], &dst4[k * kAccThreads + threadIdx.x]);
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
//
// Two shapes, chosen by whether counts fits the memory-side cache (STREAM):
//  - larger (measured on 8 matrices of 100,000 x 1,000, fraction of 8 TB/s on
//    (4K + 8) bytes per cell): one-wavefront workgroups that walk 1 KiB tiles,
//    four to twelve per compute unit, every group of counts written back whether or not
//    its sum is zero, counts accessed with the no-reuse hint: 0.74.  Writing
//    back only the groups whose sum is not zero saves a quarter of the written
//    bytes and costs 8 %: what reaches memory are then lines written in pieces.
//    With 1,024-lane workgroups (two per compute unit) the same kernel runs at
//    0.67, with the conditional write-back and plain accesses at 0.63; 2 or 4
//    groups per lane: 0.66-0.71;
//  - smaller: 1,024-lane workgroups, two groups per lane, up to 2,048 of them,
//    plain accesses, groups with a zero sum not written (the lines stay in the
//    cache, where pieces merge): a 10,000 x 1,000 matrix takes 74 us against
//    85 us in the other shape, 1,000 x 1,000 10 us against 19 us.
// ---------------------------------------------------------------------------
constexpr int kDeltaChunk = 8;              // delta matrices whose loads are in flight together
constexpr unsigned kDeltaMaxGrid = 2048;    // otherwise: workgroups of the persistent grid
constexpr unsigned long long kDeltaCachedBytes = 256ull << 20;     // counts up to this size are left cacheable

// STREAM: workgroups of the persistent grid per compute unit, by the number of
// delta matrices (100,000 x 1,000 cells; fraction of 8 TB/s with 4, 6, 8, 12 per
// unit: K = 1: 0.41 0.54 0.62 0.64; K = 2: 0.50 0.65 0.71 0.69; K = 4: 0.64 0.76
// 0.74 0.71; K = 8: 0.74 0.72 0.72 0.67; K = 12: 0.68 0.71 0.72 0.67; K = 16:
// 0.72 0.71 0.71 0.67; K = 32: 0.70 0.71 0.71 0.68).
inline unsigned delta_per_cu(int K)
{
    if (K == 1) return 12;
    if (K <= 3) return 8;
    return K == 8 || K == 16 ? 4 : 6;
}

template <bool STREAM>
struct DeltaShape {
    static constexpr int kThreads = STREAM ? 64 : 1024;     // lanes of a workgroup
    static constexpr int kVpt = STREAM ? 1 : 2;             // 128-bit groups per lane and step
};

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

template <bool LDS_TOTALS, bool STREAM>
__global__ __launch_bounds__(DeltaShape<STREAM>::kThreads) void dense_delta_kernel(const DeltaArgs a)
{
    constexpr int kDeltaThreads = DeltaShape<STREAM>::kThreads, kDeltaVpt = DeltaShape<STREAM>::kVpt;
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
    // deltas (not after their sum is known), so that the latencies overlap.
    // STREAM: every group is written back, so that whole lines reach the memory.
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
            old[v] = !on[v] ? u32x4{0, 0, 0, 0} : STREAM ? __builtin_nontemporal_load(&counts4[g]) : counts4[g];
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
            if (!on[v]) continue;
            const unsigned long long g = g0 + static_cast<unsigned long long>(v) * kDeltaThreads;
            const bool changed = (sum[v].x | sum[v].y | sum[v].z | sum[v].w) != 0;
            if constexpr (STREAM) {
                __builtin_nontemporal_store(old[v] + sum[v], &counts4[g]);
            } else {
                if (changed) counts4[g] = old[v] + sum[v];
            }
            if (changed) {
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

// Words cleared before every call: sampled histogram and padded cursors.
size_t zeroed_words(uint32_t n_tiles) { return n_tiles + static_cast<size_t>(kCursorStride) * (kMaxCoarse + n_tiles); }

// Upper bounds of the work lists the plan kernel builds on the device: the sum
// over groups of ceil(room_g / step) is at most slots / step + number of groups.
size_t max_fine_steps(size_t slots, uint32_t n_coarse) { return slots / kPartTile + n_coarse; }
size_t max_acc_items(size_t slots, uint32_t n_tiles) { return slots / kAccChunk + n_tiles; }

// Every how many blocks of kSampleBlock triples one is sampled.
long long sample_period(long long n, uint32_t n_tiles)
{
    long long period = n / (kSamplePerTile * static_cast<long long>(n_tiles));
    if (period > kSampleMaxPeriod) period = kSampleMaxPeriod;
    return period < 1 ? 1 : period;
}

// Words of tmp and of sorted: the rooms of all tiles add up to at most
//   (S + kRoomSigmas * sqrt(tiles * S) + kRoomFloor * tiles) * n / S + tiles
// for a sample of S triples (Cauchy-Schwarz on the square roots).  S is not
// known here (it depends on how the triples are spread over the buffers), but
// the bound falls as S grows, and S >= n / (2 * period): a buffer of m triples
// has ceil(ceil(m / 256) / period) sampled blocks, all full but the last.
size_t slots_for(long long n, uint32_t n_tiles, long long period)
{
    // (at least one sampled triple; a buffer shorter than one block is sampled whole)
    const double least = n / (2.0 * static_cast<double>(period)) < 1.0 ? 1.0 : n / (2.0 * static_cast<double>(period));
    const double tiles = n_tiles;
    double bound = (least + kRoomSigmas * __builtin_sqrt(tiles * least) + kRoomFloor * tiles) * (n / least) + tiles;
    bound = bound * 1.001 + 1024.0;                      // rounding of the kernel's binary32 arithmetic
    const double most = 2147483647.0 - 256.0;            // sorted_base + n_slots stays below 2^32 - 1
    return static_cast<size_t>(bound < most ? bound : most);
}

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
    const size_t n_slots = slots_for(n, n_tiles, sample_period(n, n_tiles));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = ws != nullptr ? ws + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    // hist, coarse_cursor, fine_cursor are contiguous: cleared by one kernel.
    char *hist = take(sizeof(uint32_t) * zeroed_words(n_tiles));
    char *tile_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *coarse_part_start = take(sizeof(uint32_t) * (n_coarse + 1));
    char *chunk_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *hot_chunk_start = take(sizeof(uint32_t) * (kMaxCoarse + 1));
    char *hot_tile = take(sizeof(uint32_t) * kMaxCoarse);
    char *tmp_start = take(sizeof(uint32_t) * (n_coarse + 1));
    char *digit_start = take(sizeof(uint32_t) * kMaxCoarse);
    char *digit_room = take(sizeof(uint32_t) * kMaxCoarse);
    char *tile_digit = take((static_cast<size_t>(n_tiles) + 3) / 4 * 4);     // whole words
    const size_t tmp_at = off;
    char *tmp = take(sizeof(uint32_t) * n_slots);
    const size_t sorted_at = off;
    char *sorted = take(sizeof(uint32_t) * n_slots);
    if (plan != nullptr) {
        plan->hist = reinterpret_cast<uint32_t *>(hist);
        plan->coarse_cursor = plan->hist + n_tiles;
        plan->fine_cursor = plan->coarse_cursor + static_cast<size_t>(kCursorStride) * kMaxCoarse;
        plan->tile_start = reinterpret_cast<uint32_t *>(tile_start);
        plan->coarse_part_start = reinterpret_cast<uint32_t *>(coarse_part_start);
        plan->chunk_start = reinterpret_cast<uint32_t *>(chunk_start);
        plan->hot_chunk_start = reinterpret_cast<uint32_t *>(hot_chunk_start);
        plan->hot_tile = reinterpret_cast<uint32_t *>(hot_tile);
        plan->tmp_start = reinterpret_cast<uint32_t *>(tmp_start);
        plan->digit_start = reinterpret_cast<uint32_t *>(digit_start);
        plan->digit_room = reinterpret_cast<uint32_t *>(digit_room);
        plan->tile_digit = reinterpret_cast<uint8_t *>(tile_digit);
        plan->tmp = reinterpret_cast<uint32_t *>(tmp);
        plan->sorted = reinterpret_cast<uint32_t *>(sorted);
        plan->sorted_base = static_cast<uint32_t>((sorted_at - tmp_at) / sizeof(uint32_t));
        plan->n_tiles = n_tiles;
        plan->n_coarse = n_coarse;
        plan->n_slots = static_cast<uint32_t>(n_slots);
        plan->per_sampled = 1.0f;
        plan->n_cells = cells;
    }
    return off;
}

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
    a.n_buffers = used;
    a.sample_period = 1;
    for (int k = 0; k <= MLF_MAX_K; ++k) a.step_start[k] = a.sample_start[k] = 0;
    hipStream_t s = static_cast<hipStream_t>(stream);

    BinPlan plan = {};
    const size_t need = plan_layout(V, T, total, static_cast<char *>(workspace), &plan);
    const bool binned = need != 0 && workspace != nullptr && workspace_bytes >= need &&
                        reinterpret_cast<uintptr_t>(workspace) % 256 == 0;
    if (!binned) {
        // Enough workgroups to fill the chip, few enough that their merges of
        // private totals stay small next to the streamed triples.
        long long per_buffer = (longest + kScanBlock * 16 - 1) / (kScanBlock * 16);
        const long long cap = (kScanWorkgroups + used - 1) / used;
        if (per_buffer > cap) per_buffer = cap;
        if (per_buffer < 1) per_buffer = 1;
        const dim3 grid(static_cast<unsigned>(per_buffer), static_cast<unsigned>(used));
        const bool lds_totals = totals != nullptr && T <= kMaxLdsTopics;
        const bool ok = lds_totals ? launch_kernel(direct_kernel<true>, grid, dim3(kScanBlock),
                                                   static_cast<size_t>(T) * sizeof(int32_t), s, a)
                                   : launch_kernel(direct_kernel<false>, grid, dim3(kScanBlock), 0, s, a);
        return ok ? MLF_OK : MLF_EHIP;
    }

    // The sample and the steps of the coarse level.
    const long long period = sample_period(total, plan.n_tiles);
    a.sample_period = static_cast<int>(period);
    long long sampled = 0;
    for (int k = 0; k < used; ++k) {
        const long long m = a.n_triples[k];
        const long long blocks = (m + kSampleBlock - 1) / kSampleBlock;
        const long long picked = (blocks + period - 1) / period;          // blocks 0, period, 2 period, ...
        const long long last = (picked - 1) * period;                     // the last one may be short
        sampled += (picked - 1) * kSampleBlock + (m - last * kSampleBlock < kSampleBlock ? m - last * kSampleBlock : kSampleBlock);
        a.step_start[k + 1] = a.step_start[k] + static_cast<uint32_t>((m + kPartTile - 1) / kPartTile);
        a.sample_start[k + 1] = a.sample_start[k] + static_cast<uint32_t>(picked);
    }
    for (int k = used + 1; k <= MLF_MAX_K; ++k) {
        a.step_start[k] = a.step_start[used];
        a.sample_start[k] = a.sample_start[used];
    }
    plan.per_sampled = static_cast<float>(static_cast<double>(total) / static_cast<double>(sampled));

    // 1. clear the counters, 2. sample histogram, 3. room and offsets,
    // 4. coarse partition (+ totals, rejects), 5. fine partition, 6. accumulate and merge.
    const uint32_t n_clear = static_cast<uint32_t>(zeroed_words(plan.n_tiles));
    if (!launch_kernel(clear_kernel, dim3((n_clear + kThreads - 1) / kThreads), dim3(kThreads), 0, s,
                       plan.hist, n_clear)) {
        return MLF_EHIP;
    }
    const size_t hist_lds = static_cast<size_t>(plan.n_tiles) * sizeof(uint32_t);
    const long long per_workgroup = (kScanBlock / kSampleBlock) * kSampleUnroll;
    long long sample_grid = (a.sample_start[used] + per_workgroup - 1) / per_workgroup;
    if (sample_grid > kSampleWorkgroups) sample_grid = kSampleWorkgroups;
    if (sample_grid < 1) sample_grid = 1;
    const bool sampled_ok =
        hist_lds <= 65536 ? launch_kernel(sample_kernel<false>, dim3(static_cast<unsigned>(sample_grid)),
                                          dim3(kScanBlock), hist_lds, s, a, plan)
                          : launch_kernel(sample_kernel<true>, dim3(static_cast<unsigned>(sample_grid)),
                                          dim3(kScanBlock), 0, s, a, plan);
    if (!sampled_ok) return MLF_EHIP;
    if (!launch_kernel(plan_kernel, dim3(1), dim3(kPlanThreads), 0, s, plan)) return MLF_EHIP;
    const uint32_t n_steps = a.step_start[used];
    const unsigned coarse_grid = n_steps < kCoarseWorkgroups ? n_steps : kCoarseWorkgroups;
    const size_t hot_lds = static_cast<size_t>((plan.n_tiles + 3) / 4) * sizeof(uint32_t);   // digit of every tile
    const bool lds_totals = totals != nullptr && T <= kCoarseLdsTopics;
    const bool coarse_ok =
        lds_totals ? launch_kernel(coarse_partition_kernel<true>, dim3(coarse_grid), dim3(kPartThreads),
                                   hot_lds + static_cast<size_t>(T) * sizeof(int32_t), s, a, plan)
                   : launch_kernel(coarse_partition_kernel<false>, dim3(coarse_grid), dim3(kPartThreads),
                                   hot_lds, s, a, plan);
    if (!coarse_ok) return MLF_EHIP;
    const unsigned fine_steps = static_cast<unsigned>(max_fine_steps(plan.n_slots, plan.n_coarse));
    if (!launch_kernel(fine_partition_kernel, dim3(fine_steps), dim3(kPartThreads), 0, s, counts, plan)) return MLF_EHIP;
    const unsigned acc_items = static_cast<unsigned>(max_acc_items(plan.n_slots, plan.n_tiles));
    if (!launch_kernel(accumulate_kernel, dim3(acc_items), dim3(kAccThreads), 0, s, counts, plan)) return MLF_EHIP;
    return MLF_OK;
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
    hipStream_t s = static_cast<hipStream_t>(stream);
    const bool lds_totals = totals != nullptr && T <= kMaxLdsTopics;
    const bool streamed = bytes > kDeltaCachedBytes;
    const unsigned threads = streamed ? DeltaShape<true>::kThreads : DeltaShape<false>::kThreads;
    const unsigned per_step = threads * (streamed ? DeltaShape<true>::kVpt : DeltaShape<false>::kVpt);
    unsigned long long tiles = (work + per_step - 1) / per_step;
    const unsigned cus = cu_count();
    const unsigned long long grid_max =
        streamed ? static_cast<unsigned long long>(cus > 0 ? cus : 256) * delta_per_cu(K) : kDeltaMaxGrid;
    if (tiles > grid_max) tiles = grid_max;
    if (tiles < 1) tiles = 1;
    const dim3 grid(static_cast<unsigned>(tiles)), block(threads);
    const size_t lds = lds_totals ? static_cast<size_t>(T) * sizeof(int32_t) : 0;
    const bool ok = lds_totals ? (streamed ? launch_kernel(dense_delta_kernel<true, true>, grid, block, lds, s, a)
                                           : launch_kernel(dense_delta_kernel<true, false>, grid, block, lds, s, a))
                               : (streamed ? launch_kernel(dense_delta_kernel<false, true>, grid, block, lds, s, a)
                                           : launch_kernel(dense_delta_kernel<false, false>, grid, block, lds, s, a));
    return ok ? MLF_OK : MLF_EHIP;
}
