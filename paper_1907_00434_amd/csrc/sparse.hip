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
// of counts[] they fall into (a two-level counting sort: 64 fine tiles per
// coarse range, so that every partition step writes long contiguous runs).
// One workgroup then owns a tile at a time: it accumulates the tile's records
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
constexpr int kTileBits = 15;                    // cells per LDS image: 32768 (128 KiB)
constexpr uint32_t kTileCells = 1u << kTileBits;
constexpr int kFineBits = 6;                     // fine tiles per coarse range: 64
constexpr uint32_t kFinePerCoarse = 1u << kFineBits;
constexpr uint32_t kMaxCoarse = 256;             // coarse ranges (one counter per lane)
constexpr uint32_t kMaxTiles = kMaxCoarse * kFinePerCoarse;   // 16384 tiles = 2^29 cells
constexpr int kPartItems = 16;                   // records per lane in a partition step
constexpr uint32_t kPartTile = kThreads * kPartItems;          // 4096 records
constexpr int kAccThreads = 1024;                // lanes of an accumulate workgroup
constexpr uint32_t kAccChunk = 1u << 16;         // records per accumulate work item
constexpr int kScanThreads = 1024;
constexpr int kScanItems = kMaxTiles / kScanThreads;           // 16
constexpr long long kMinBinnedTriples = 1 << 16; // below this the direct path is cheaper

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

// Control block of the binned path, carved out of the caller's scratch.
struct BinPlan {
    uint32_t *hist;               // [n_tiles]   records per tile            (zeroed)
    uint32_t *coarse_cursor;      // [n_coarse]  records placed so far       (zeroed)
    uint32_t *fine_cursor;        // [n_tiles]   records placed so far       (zeroed)
    uint32_t *tile_start;         // [n_tiles+1] exclusive scan of hist
    uint32_t *coarse_part_start;  // [n_coarse+1] partition steps before each coarse range
    uint32_t *chunk_start;        // [n_tiles+1] accumulate work items before each tile
    Record *tmp;                  // [n] grouped by coarse range
    Record *sorted;               // [n] grouped by tile
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

// First pass over the triples; blockIdx.y = worker buffer, blockIdx.x strides
// over that buffer.  BINNED = false: the direct path (counts[] updated here).
// BINNED = true: only the per-tile histogram is built.  Both keep the totals in
// LDS and count the rejected triples.
// Dynamic LDS: [T totals if LDS_TOTALS][n_tiles histogram if BINNED].
template <bool BINNED, bool LDS_TOTALS>
__global__ __launch_bounds__(kThreads) void scan_triples_kernel(const SparseArgs a,
                                                                const BinPlan plan)
{
    extern __shared__ int32_t lds[];
    const int T = a.T;
    const bool want_totals = a.totals != nullptr;
    int32_t *lds_totals = lds;
    uint32_t *lds_hist = reinterpret_cast<uint32_t *>(lds + (LDS_TOTALS ? T : 0));
    if constexpr (LDS_TOTALS) {
        for (int t = threadIdx.x; t < T; t += kThreads) lds_totals[t] = 0;
    }
    if constexpr (BINNED) {
        for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kThreads) lds_hist[b] = 0;
    }
    if constexpr (LDS_TOTALS || BINNED) __syncthreads();

    const int k = blockIdx.y;
    const int32_t *tr = a.triples[k];
    const long long m = a.n_triples[k];
    const long long stride = static_cast<long long>(gridDim.x) * kThreads;
    int n_bad = 0;
    for (long long r = static_cast<long long>(blockIdx.x) * kThreads + threadIdx.x; r < m;
         r += stride) {
        int word, topic, delta;
        if (!load_triple(tr, r, a.V, T, word, topic, delta)) {
            ++n_bad;
            continue;
        }
        const long long cell = static_cast<long long>(word) * T + topic;
        if constexpr (BINNED) {
            lds_fetch_add(&lds_hist[static_cast<uint32_t>(cell) >> kTileBits], 1u);
        } else {
            add_relaxed(a.counts + cell, delta);
        }
        if (want_totals) {
            if constexpr (LDS_TOTALS) {
                lds_add(&lds_totals[topic], delta);
            } else {
                add_relaxed(a.totals + topic, delta);
            }
        }
    }

    if constexpr (LDS_TOTALS || BINNED) __syncthreads();
    if constexpr (LDS_TOTALS) {
        if (want_totals) {
            for (int t = threadIdx.x; t < T; t += kThreads) {
                const int32_t v = lds_totals[t];
                if (v != 0) add_relaxed(a.totals + t, v);
            }
        }
    }
    if constexpr (BINNED) {
        for (uint32_t b = threadIdx.x; b < plan.n_tiles; b += kThreads) {
            const uint32_t v = lds_hist[b];
            if (v != 0) fetch_add_relaxed(plan.hist + b, v);
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

// Exclusive prefix sum over up to kMaxTiles values with one workgroup of
// kScanThreads lanes: lane i owns kScanItems consecutive values.
// `value(j)` gives input j; out[j] receives the sum of inputs before j and
// out[n] the total.  `scratch` is kScanThreads words of LDS.
template <typename F>
__device__ void block_exclusive_scan(uint32_t n, F value, uint32_t *out, uint32_t *scratch)
{
    const uint32_t first = threadIdx.x * kScanItems;
    uint32_t local[kScanItems];
    uint32_t sum = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        const uint32_t j = first + i;
        local[i] = j < n ? value(j) : 0u;
        sum += local[i];
    }
    scratch[threadIdx.x] = sum;
    __syncthreads();
    // Hillis-Steele scan of the kScanThreads partial sums.
    for (int off = 1; off < kScanThreads; off <<= 1) {
        const uint32_t add = threadIdx.x >= static_cast<uint32_t>(off) ? scratch[threadIdx.x - off] : 0u;
        __syncthreads();
        scratch[threadIdx.x] += add;
        __syncthreads();
    }
    uint32_t run = scratch[threadIdx.x] - sum;     // exclusive prefix of this lane
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        const uint32_t j = first + i;
        if (j < n) out[j] = run;
        run += local[i];
    }
    if (threadIdx.x == kScanThreads - 1) out[n] = scratch[kScanThreads - 1];
    __syncthreads();
}

// One workgroup: turns the tile histogram into the offsets every later step uses.
__global__ __launch_bounds__(kScanThreads) void plan_kernel(const BinPlan plan)
{
    __shared__ uint32_t scratch[kScanThreads];
    const uint32_t *hist = plan.hist;
    block_exclusive_scan(plan.n_tiles, [=](uint32_t j) { return hist[j]; }, plan.tile_start,
                         scratch);
    __threadfence_block();
    const uint32_t *tile_start = plan.tile_start;
    const uint32_t n_tiles = plan.n_tiles;
    // Partition steps (kPartTile records each) per coarse range.
    block_exclusive_scan(
        plan.n_coarse,
        [=](uint32_t c) {
            const uint32_t lo = c << kFineBits;
            const uint32_t hi = min(lo + kFinePerCoarse, n_tiles);
            const uint32_t cnt = tile_start[hi] - tile_start[lo];
            return (cnt + kPartTile - 1) / kPartTile;
        },
        plan.coarse_part_start, scratch);
    // Accumulate work items (kAccChunk records each) per tile.
    block_exclusive_scan(
        n_tiles, [=](uint32_t j) { return (hist[j] + kAccChunk - 1) / kAccChunk; },
        plan.chunk_start, scratch);
}

// Largest index i in [0, n) with start[i] <= g, for a non-decreasing start[] with
// start[0] = 0 and g < start[n].
__device__ __forceinline__ uint32_t owner_of(const uint32_t *start, uint32_t n, uint32_t g)
{
    uint32_t lo = 0, hi = n;
    while (hi - lo > 1) {
        const uint32_t mid = (lo + hi) >> 1;
        if (start[mid] <= g) {
            lo = mid;
        } else {
            hi = mid;
        }
    }
    return lo;
}

// One partition step of a workgroup: up to kPartTile records held in registers
// are grouped by `digit` (n_digits <= kThreads) in LDS and written out so that
// the records of one digit form one contiguous run at the place reserved for
// them in the output.
//   rec[i], live[i]  the lane's records and whether each exists
//   digit_of(cell)   digit of a record
//   reserve(d, n)    output index where this step's n records of digit d go
struct PartitionLds {
    Record stage[kPartTile];
    uint32_t count[kThreads];
    uint32_t offset[kThreads];
    uint32_t dest[kThreads];
};

template <typename DigitOf, typename Reserve>
__device__ __forceinline__ void partition_step(PartitionLds &s, const Record (&rec)[kPartItems],
                                               const bool (&live)[kPartItems], uint32_t n_digits,
                                               DigitOf digit_of, Reserve reserve, Record *out)
{
    s.count[threadIdx.x] = 0;
    __syncthreads();
    uint32_t rank[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        rank[i] = live[i] ? lds_fetch_add(&s.count[digit_of(rec[i].cell)], 1u) : 0u;
    }
    __syncthreads();
    // Exclusive scan of the digit counts: one digit per lane.
    const uint32_t mine = threadIdx.x < n_digits ? s.count[threadIdx.x] : 0u;
    s.offset[threadIdx.x] = mine;
    __syncthreads();
    for (int off = 1; off < kThreads; off <<= 1) {
        const uint32_t add = threadIdx.x >= static_cast<uint32_t>(off) ? s.offset[threadIdx.x - off] : 0u;
        __syncthreads();
        s.offset[threadIdx.x] += add;
        __syncthreads();
    }
    const uint32_t total = s.offset[kThreads - 1];
    __syncthreads();
    s.offset[threadIdx.x] -= mine;                      // inclusive -> exclusive
    if (mine != 0) s.dest[threadIdx.x] = reserve(threadIdx.x, mine);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        if (live[i]) s.stage[s.offset[digit_of(rec[i].cell)] + rank[i]] = rec[i];
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < total; i += kThreads) {
        const Record r = s.stage[i];
        const uint32_t d = digit_of(r.cell);
        out[s.dest[d] + (i - s.offset[d])] = r;
    }
}

// Coarse partition: blockIdx.y = worker buffer, blockIdx.x = step within it.
// Valid triples become records in plan.tmp, grouped by coarse range.
__global__ __launch_bounds__(kThreads) void coarse_partition_kernel(const SparseArgs a,
                                                                    const BinPlan plan)
{
    __shared__ PartitionLds s;
    const int32_t *tr = a.triples[blockIdx.y];
    const long long m = a.n_triples[blockIdx.y];
    const long long base = static_cast<long long>(blockIdx.x) * kPartTile;
    if (base >= m) return;                               // uniform for the workgroup
    Record rec[kPartItems];
    bool live[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        const long long r = base + i * kThreads + threadIdx.x;
        int word = 0, topic = 0, delta = 0;
        live[i] = r < m && load_triple(tr, r, a.V, a.T, word, topic, delta);
        rec[i].cell = static_cast<uint32_t>(static_cast<long long>(word) * a.T + topic);
        rec[i].delta = delta;
    }
    const uint32_t *tile_start = plan.tile_start;
    uint32_t *cursor = plan.coarse_cursor;
    partition_step(
        s, rec, live, plan.n_coarse,
        [](uint32_t cell) { return cell >> (kTileBits + kFineBits); },
        [=](uint32_t c, uint32_t n) {
            return tile_start[c << kFineBits] + fetch_add_relaxed(cursor + c, n);
        },
        plan.tmp);
}

// Fine partition: workgroup g takes one step of one coarse range of plan.tmp
// and writes its records to plan.sorted, grouped by tile.
__global__ __launch_bounds__(kThreads) void fine_partition_kernel(const BinPlan plan)
{
    __shared__ PartitionLds s;
    __shared__ uint32_t s_coarse;
    const uint32_t g = blockIdx.x;
    if (g >= plan.coarse_part_start[plan.n_coarse]) return;   // uniform
    if (threadIdx.x == 0) s_coarse = owner_of(plan.coarse_part_start, plan.n_coarse, g);
    __syncthreads();
    const uint32_t c = s_coarse;
    const uint32_t first_tile = c << kFineBits;
    const uint32_t last_tile = min(first_tile + kFinePerCoarse, plan.n_tiles);
    const uint32_t begin = plan.tile_start[first_tile] + (g - plan.coarse_part_start[c]) * kPartTile;
    const uint32_t end = min(begin + kPartTile, plan.tile_start[last_tile]);
    Record rec[kPartItems];
    bool live[kPartItems];
#pragma unroll
    for (int i = 0; i < kPartItems; ++i) {
        const uint32_t r = begin + i * kThreads + threadIdx.x;
        live[i] = r < end;
        rec[i] = live[i] ? plan.tmp[r] : Record{0u, 0};
    }
    const uint32_t *tile_start = plan.tile_start;
    uint32_t *cursor = plan.fine_cursor;
    partition_step(
        s, rec, live, kFinePerCoarse,
        [](uint32_t cell) { return (cell >> kTileBits) & (kFinePerCoarse - 1); },
        [=](uint32_t f, uint32_t n) {
            const uint32_t tile = first_tile + f;
            return tile_start[tile] + fetch_add_relaxed(cursor + tile, n);
        },
        plan.sorted);
}

// Accumulate: workgroup g takes up to kAccChunk records of one tile, sums them
// into a private LDS image of the tile and merges the image into counts[].
__global__ __launch_bounds__(kAccThreads) void accumulate_kernel(int32_t *counts,
                                                                 const BinPlan plan)
{
    __shared__ int32_t image[kTileCells];
    __shared__ uint32_t s_tile;
    const uint32_t g = blockIdx.x;
    if (g >= plan.chunk_start[plan.n_tiles]) return;          // uniform
    if (threadIdx.x == 0) s_tile = owner_of(plan.chunk_start, plan.n_tiles, g);
    for (uint32_t i = threadIdx.x; i < kTileCells; i += kAccThreads) image[i] = 0;
    __syncthreads();
    const uint32_t tile = s_tile;
    const uint32_t chunks = plan.chunk_start[tile + 1] - plan.chunk_start[tile];
    const uint32_t begin = plan.tile_start[tile] + (g - plan.chunk_start[tile]) * kAccChunk;
    const uint32_t end = min(begin + kAccChunk, plan.tile_start[tile + 1]);
    for (uint32_t r = begin + threadIdx.x; r < end; r += kAccThreads) {
        const Record rec = plan.sorted[r];
        lds_add(&image[rec.cell & (kTileCells - 1)], rec.delta);
    }
    __syncthreads();
    const unsigned long long base = static_cast<unsigned long long>(tile) << kTileBits;
    const unsigned long long left = plan.n_cells - base;
    const uint32_t cells = left < kTileCells ? static_cast<uint32_t>(left) : kTileCells;
    int32_t *dst = counts + base;
    if (chunks == 1) {
        // This workgroup is the only writer of the tile: plain read-modify-write.
        for (uint32_t i = threadIdx.x; i < cells; i += kAccThreads) {
            const int32_t v = image[i];
            if (v != 0) dst[i] = static_cast<int32_t>(static_cast<uint32_t>(dst[i]) + static_cast<uint32_t>(v));
        }
    } else {
        for (uint32_t i = threadIdx.x; i < cells; i += kAccThreads) {
            const int32_t v = image[i];
            if (v != 0) add_relaxed(dst + i, v);
        }
    }
}

// ---------------------------------------------------------------------------
// Host side.
// ---------------------------------------------------------------------------

size_t align_up(size_t x) { return (x + 255) & ~static_cast<size_t>(255); }

// Whether the binned path can serve this shape, and its scratch layout.
// Returns the scratch size in bytes (0 when the shape is not eligible).
size_t plan_layout(int32_t V, int32_t T, long long n, char *ws, BinPlan *plan)
{
    if (V < 1 || T < 1 || n < 1 || n > 0x7fffffffll) return 0;
    const unsigned long long cells = static_cast<unsigned long long>(V) * static_cast<unsigned long long>(T);
    const unsigned long long tiles = (cells + kTileCells - 1) >> kTileBits;
    if (tiles > kMaxTiles) return 0;
    const uint32_t n_tiles = static_cast<uint32_t>(tiles);
    const uint32_t n_coarse = (n_tiles + kFinePerCoarse - 1) >> kFineBits;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *p = ws != nullptr ? ws + off : nullptr;
        off += align_up(bytes);
        return p;
    };
    // hist, coarse_cursor, fine_cursor are contiguous: cleared by one kernel.
    char *hist = take(sizeof(uint32_t) * (2 * static_cast<size_t>(n_tiles) + n_coarse));
    char *tile_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *coarse_part_start = take(sizeof(uint32_t) * (n_coarse + 1));
    char *chunk_start = take(sizeof(uint32_t) * (n_tiles + 1));
    char *tmp = take(sizeof(Record) * static_cast<size_t>(n));
    char *sorted = take(sizeof(Record) * static_cast<size_t>(n));
    if (plan != nullptr) {
        plan->hist = reinterpret_cast<uint32_t *>(hist);
        plan->coarse_cursor = plan->hist + n_tiles;
        plan->fine_cursor = plan->coarse_cursor + n_coarse;
        plan->tile_start = reinterpret_cast<uint32_t *>(tile_start);
        plan->coarse_part_start = reinterpret_cast<uint32_t *>(coarse_part_start);
        plan->chunk_start = reinterpret_cast<uint32_t *>(chunk_start);
        plan->tmp = reinterpret_cast<Record *>(tmp);
        plan->sorted = reinterpret_cast<Record *>(sorted);
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
    if (total_triples < kMinBinnedTriples) return 0;
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
    long long per_buffer = (longest + kThreads * 16 - 1) / (kThreads * 16);
    const long long cap = (2048 + used - 1) / used;
    if (per_buffer > cap) per_buffer = cap;
    if (per_buffer < 1) per_buffer = 1;
    const dim3 scan_grid(static_cast<unsigned>(per_buffer), static_cast<unsigned>(used));
    bool lds_totals = totals != nullptr && T <= kMaxLdsTopics;
    size_t totals_lds = lds_totals ? static_cast<size_t>(T) * sizeof(int32_t) : 0;

    BinPlan plan = {};
    const size_t need = total >= kMinBinnedTriples
                            ? plan_layout(V, T, total, static_cast<char *>(workspace), &plan)
                            : 0;
    const bool binned = need != 0 && workspace != nullptr && workspace_bytes >= need &&
                        reinterpret_cast<uintptr_t>(workspace) % 256 == 0;
    if (!binned) {
        if (lds_totals) {
            scan_triples_kernel<false, true><<<scan_grid, dim3(kThreads), totals_lds, s>>>(a, plan);
        } else {
            scan_triples_kernel<false, false><<<scan_grid, dim3(kThreads), 0, s>>>(a, plan);
        }
        return launched() ? MLF_OK : MLF_EHIP;
    }

    // 1. clear the counters, 2. histogram (+ totals, rejects), 3. offsets,
    // 4. coarse partition, 5. fine partition, 6. accumulate and merge.
    const uint32_t n_clear = 2 * plan.n_tiles + plan.n_coarse;
    clear_kernel<<<dim3((n_clear + kThreads - 1) / kThreads), dim3(kThreads), 0, s>>>(plan.hist, n_clear);
    if (!launched()) return MLF_EHIP;
    const size_t hist_lds = static_cast<size_t>(plan.n_tiles) * sizeof(uint32_t);
    if (totals_lds + hist_lds > 65536) {    // keep the first pass within 64 KiB of LDS
        lds_totals = false;
        totals_lds = 0;
    }
    if (lds_totals) {
        scan_triples_kernel<true, true><<<scan_grid, dim3(kThreads), totals_lds + hist_lds, s>>>(a, plan);
    } else {
        scan_triples_kernel<true, false><<<scan_grid, dim3(kThreads), hist_lds, s>>>(a, plan);
    }
    if (!launched()) return MLF_EHIP;
    plan_kernel<<<dim3(1), dim3(kScanThreads), 0, s>>>(plan);
    if (!launched()) return MLF_EHIP;
    const unsigned steps_per_buffer = static_cast<unsigned>((longest + kPartTile - 1) / kPartTile);
    coarse_partition_kernel<<<dim3(steps_per_buffer, static_cast<unsigned>(used)), dim3(kThreads), 0, s>>>(a, plan);
    if (!launched()) return MLF_EHIP;
    // Upper bounds of the work lists the plan kernel builds on the device:
    // ceil(n_c / tile) summed over ranges <= n / tile + number of ranges.
    const unsigned fine_steps = static_cast<unsigned>(total / kPartTile) + plan.n_coarse;
    fine_partition_kernel<<<dim3(fine_steps), dim3(kThreads), 0, s>>>(plan);
    if (!launched()) return MLF_EHIP;
    const unsigned acc_items = static_cast<unsigned>(total / kAccChunk) + plan.n_tiles;
    accumulate_kernel<<<dim3(acc_items), dim3(kAccThreads), 0, s>>>(counts, plan);
    return launched() ? MLF_OK : MLF_EHIP;
}
