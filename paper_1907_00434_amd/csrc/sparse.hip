// LDA count-delta scatter-add for gfx950 (Sec. 6 of the paper: a worker's LDA
// update is a numerical update to the word-topic count matrix).
//
// Direct path: every workgroup streams a slice of one worker's triple buffer,
// adds the deltas into counts[] with device-scope integer atomics, and keeps a
// private copy of the per-topic totals in LDS that it merges into totals[] once
// at the end, so that the T-entry totals vector -- which every triple hits --
// never sees per-triple global atomics.  Integer addition commutes, so any
// interleaving gives the same bits.
#include <hip/hip_runtime.h>

#include <stdint.h>

#include "mlfabric.h"

namespace {

constexpr int kThreads = 256;
constexpr int kMaxLdsTopics = 16384;   // totals privatised in LDS up to 64 KiB

struct SparseArgs {
    const int32_t *triples[MLF_MAX_K];
    long long n_triples[MLF_MAX_K];
    int32_t *counts;
    int32_t *totals;
    int32_t *rejected;
    int V;
    int T;
};

struct Triple {
    int32_t word, topic, delta;
};

__device__ __forceinline__ void add_relaxed(int32_t *p, int32_t v)
{
    __hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// blockIdx.y = worker buffer, blockIdx.x strides over that buffer's triples.
template <bool LDS_TOTALS>
__global__ __launch_bounds__(kThreads) void scatter_direct_kernel(const SparseArgs a)
{
    extern __shared__ int32_t lds_totals[];
    const int T = a.T;
    const bool want_totals = a.totals != nullptr;
    if constexpr (LDS_TOTALS) {
        if (want_totals) {
            for (int t = threadIdx.x; t < T; t += kThreads) lds_totals[t] = 0;
        }
        __syncthreads();
    }

    const int k = blockIdx.y;
    const int32_t *tr = a.triples[k];
    const long long m = a.n_triples[k];
    const long long stride = static_cast<long long>(gridDim.x) * kThreads;
    int n_bad = 0;
    for (long long r = static_cast<long long>(blockIdx.x) * kThreads + threadIdx.x; r < m;
         r += stride) {
        Triple t;   // read once: streaming loads
        t.word = __builtin_nontemporal_load(tr + 3 * r);
        t.topic = __builtin_nontemporal_load(tr + 3 * r + 1);
        t.delta = __builtin_nontemporal_load(tr + 3 * r + 2);
        const bool ok = static_cast<unsigned>(t.word) < static_cast<unsigned>(a.V) &&
                        static_cast<unsigned>(t.topic) < static_cast<unsigned>(T);
        if (!ok) {
            ++n_bad;
            continue;
        }
        add_relaxed(a.counts + static_cast<long long>(t.word) * T + t.topic, t.delta);
        if (want_totals) {
            if constexpr (LDS_TOTALS) {
                __hip_atomic_fetch_add(&lds_totals[t.topic], t.delta, __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_WORKGROUP);
            } else {
                add_relaxed(a.totals + t.topic, t.delta);
            }
        }
    }

    if constexpr (LDS_TOTALS) {
        __syncthreads();
        if (want_totals) {
            for (int t = threadIdx.x; t < T; t += kThreads) {
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

}  // namespace

extern "C" size_t mlf_sparse_workspace_bytes(int32_t V, int32_t T, int64_t total_triples)
{
    (void)V;
    (void)T;
    (void)total_triples;
    return 0;
}

extern "C" mlf_status mlf_sparse_scatter_add(int32_t *counts, int32_t *totals, int32_t V,
                                             int32_t T, const int32_t *const *triple_ptrs,
                                             const int64_t *n_triples, int K, void *workspace,
                                             size_t workspace_bytes, int32_t *n_rejected,
                                             mlf_stream stream)
{
    (void)workspace;
    (void)workspace_bytes;
    if (counts == nullptr || V < 1 || T < 1 || K < 0) return MLF_EINVAL;
    if (K > MLF_MAX_K) return MLF_EUNSUPPORTED;
    if (K > 0 && (triple_ptrs == nullptr || n_triples == nullptr)) return MLF_EINVAL;

    SparseArgs a;
    long long longest = 0;
    int used = 0;
    for (int k = 0; k < K; ++k) {
        if (n_triples[k] < 0) return MLF_EINVAL;
        if (n_triples[k] == 0) continue;
        if (triple_ptrs[k] == nullptr) return MLF_EINVAL;
        if (reinterpret_cast<uintptr_t>(triple_ptrs[k]) % 4 != 0) return MLF_EALIGN;
        a.triples[used] = triple_ptrs[k];
        a.n_triples[used] = n_triples[k];
        if (n_triples[k] > longest) longest = n_triples[k];
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

    // Enough workgroups to fill the chip, but few enough that the per-workgroup
    // merge of the private totals stays small next to the streamed triples.
    long long per_buffer = (longest + kThreads * 16 - 1) / (kThreads * 16);
    const long long cap = (4096 + used - 1) / used;
    if (per_buffer > cap) per_buffer = cap;
    if (per_buffer < 1) per_buffer = 1;
    const dim3 grid(static_cast<unsigned>(per_buffer), static_cast<unsigned>(used));
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (totals != nullptr && T <= kMaxLdsTopics) {
        scatter_direct_kernel<true>
            <<<grid, dim3(kThreads), static_cast<size_t>(T) * sizeof(int32_t), s>>>(a);
    } else {
        scatter_direct_kernel<false><<<grid, dim3(kThreads), 0, s>>>(a);
    }
    return hipGetLastError() == hipSuccess ? MLF_OK : MLF_EHIP;
}
