// Unified Monte-Carlo value update (Sec. 3.2, Eq. "unified update"; App. A, bandit-style update):
//   Q[id_j] <- Q[id_j] + alpha (r_j - Q[id_j])   for j = 0..M-1 in array order.
//
// Several queries of one batch often retrieve the same entry, so ids repeat, and the recursion is
// order dependent (its unrolled form in App. A weights reward k by (1-alpha)^(t-1-k)).  Instead of
// atomics on Q, every id is owned by exactly one workgroup: workgroup b of a launch reads all M ids
// and keeps those whose hash falls into bucket b, so all occurrences of an id meet in one LDS list.
// There the (id, position) pairs are sorted -- the occurrences of an id become one contiguous
// segment in array order -- and the first lane of each segment folds it sequentially and is the
// single writer of that Q entry.  fp32 with one rounding per operation (no fused multiply-add), so
// the result is the one a sequential fp32 loop reaches, bit for bit.
// The buckets need no communication (no device-wide counters, one launch), their sorts are short
// (M / buckets pairs on average), and a bucket can hold a whole launch's pairs if every id hashes
// to it (UPD_CHUNK pairs, 128 KB of LDS); the host splits longer batches into consecutive launches,
// which preserves array order.  What cannot be shortened is the fold of a long segment (a batch that
// names one id thousands of times): it is a chain of dependent roundings.
#pragma once
#include "k_select.h"
#include "layout.h"

namespace evk {

constexpr int UPD_CHUNK = 16384;          // pairs per launch
constexpr int UPD_MAX_BUCKETS = 128;      // workgroups per launch (a power of two)
constexpr int UPD_PAD = 32;               // spare list entries (read ahead by the fold, never used)

// log2 of the number of buckets used for a launch of M pairs: about 32 pairs per bucket
__host__ __device__ __forceinline__ int upd_log2_buckets(int M) {
    int lg = 0;
    while ((1 << lg) < UPD_MAX_BUCKETS && (32 << lg) < M) ++lg;
    return lg;
}

__global__ __launch_bounds__(1024) void k_update_q(const int32_t* __restrict__ ids, const float* __restrict__ rewards,
                                                   int M, float* __restrict__ qstage, int64_t N, float alpha,
                                                   uint32_t* __restrict__ counters, int log2_buckets) {
    extern __shared__ __align__(16) unsigned char upd_smem[];
    uint64_t* keys = reinterpret_cast<uint64_t*>(upd_smem);   // (id << 32 | position) while sorting, then (id, reward)
    __shared__ uint32_t n_s;
    const int tid = threadIdx.x;
    const uint32_t b = blockIdx.x;
    if (tid == 0) n_s = 0;
    __syncthreads();
    uint32_t bad = 0;
    // all of this lane's ids are requested before the first is looked at (the list insertions
    // below are memory operations the loads cannot be moved across, so a plain loop would pay
    // one memory round trip per id)
    int32_t mine[UPD_CHUNK / 1024];
#pragma unroll
    for (int u = 0; u < UPD_CHUNK / 1024; ++u) {
        const int i = tid + u * 1024;
        mine[u] = ids[i < M ? i : 0];
    }
#pragma unroll
    for (int u = 0; u < UPD_CHUNK / 1024; ++u) {
        const int i = tid + u * 1024;
        if (i >= M) continue;
        const int32_t id = mine[u];
        if (id >= 0 && (int64_t)id < N) {
            // multiplicative hash: neighbouring ids (one query's hits in one cluster) spread over the buckets
            const uint32_t h = log2_buckets ? ((uint32_t)id * 0x9E3779B1u) >> (32 - log2_buckets) : 0u;
            if (h == b) keys[atomicAdd(&n_s, 1u)] = ((uint64_t)(uint32_t)id << 32) | (uint32_t)i;
        } else {
            ++bad;
        }
    }
    if (b == 0 && bad) atomicAdd(counters, bad);   // integer diagnostic counter, not a Q value
    __syncthreads();
    const int n = (int)n_s;
    if (n == 0) return;
    int npad = 2;
    while (npad < n) npad <<= 1;
    for (int i = n + tid; i < npad; i += 1024) keys[i] = ~0ull;   // padding sorts to the end
    __syncthreads();
    // ascending sort = descending with the comparison reversed
    bitonic_desc(keys, npad, tid, 1024, [](uint64_t x, uint64_t y) { return x > y; });
    // replace positions by the rewards they point to
    for (int i = tid; i < n; i += 1024) {
        const uint64_t k = keys[i];
        keys[i] = (k & 0xffffffff00000000ull) | __float_as_uint(rewards[(uint32_t)k]);
    }
    __syncthreads();
    for (int i = tid; i < n; i += 1024) {
        const uint32_t id = (uint32_t)(keys[i] >> 32);
        if (i > 0 && (uint32_t)(keys[i - 1] >> 32) == id) continue;   // not the head of its segment
        // end of the segment: first index whose id is larger (the list is sorted), by bisection
        // (most segments have one element: look at the neighbour first)
        int lo = i + 1, hi = (i + 1 < n && (uint32_t)(keys[i + 1] >> 32) == id) ? n : i + 1;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((uint32_t)(keys[mid] >> 32) == id) lo = mid + 1; else hi = mid;
        }
        const int end = lo;
        float q = qstage[id];
        // The fold is a chain of dependent roundings.  The rewards are fetched eight at a time and one
        // batch ahead (two register sets), so that the chain never also waits for an LDS read.
        // (Reads past the segment's end are not used; the list has UPD_PAD spare entries behind it so
        // that they need no bounds check.)  The scheduler is fenced between the four parts of the
        // loop body: left alone it moves each fetch next to its fold.
        auto fetch = [&](float (&r)[8], int j) __attribute__((always_inline)) {
            const uint64_t* p = keys + j;
#pragma unroll
            for (int u = 0; u < 8; ++u) r[u] = __uint_as_float((uint32_t)p[u]);
        };
        auto fold = [&](const float (&r)[8]) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < 8; ++u) {
#pragma clang fp contract(off)   // three separately rounded operations, never a fused multiply-add
                float diff = r[u] - q;
                float stepv = alpha * diff;
                q = q + stepv;
            }
        };
        int j = i;
        if (j + 8 <= end) {
            float ra[8], rb[8];
            fetch(ra, j);
            while (j + 16 <= end) {
                fetch(rb, j + 8);
                __builtin_amdgcn_sched_barrier(0);
                fold(ra);
                __builtin_amdgcn_sched_barrier(0);
                fetch(ra, j + 16);
                __builtin_amdgcn_sched_barrier(0);
                fold(rb);
                __builtin_amdgcn_sched_barrier(0);
                j += 16;
            }
            if (j + 8 <= end) { fold(ra); j += 8; }
        }
        for (; j < end; ++j) {
#pragma clang fp contract(off)
            float diff = __uint_as_float((uint32_t)keys[j]) - q;
            float stepv = alpha * diff;
            q = q + stepv;
        }
        qstage[id] = q;
    }
}

}  // namespace evk
