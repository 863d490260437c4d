// Unified Monte-Carlo value update (Sec. 3.2, Eq. "unified update"; App. A, bandit-style update):
//   Q[id_j] <- Q[id_j] + alpha (r_j - Q[id_j])   for j = 0..M-1 in array order.
//
// Several queries of one batch often retrieve the same entry, so ids repeat, and the recursion is
// order dependent (its unrolled form in App. A weights reward k by (1-alpha)^(t-1-k)).  Instead of
// atomics, the batch is sorted by (id, position) -- all occurrences of an id become one contiguous
// segment in array order -- and the first lane of each segment folds it sequentially and is the
// single writer of that Q entry.  fp32 with one rounding per operation (no fused multiply-add), so
// the result is the one a sequential fp32 loop reaches, bit for bit.
//
// One workgroup handles up to UPD_CHUNK pairs entirely in LDS; the host splits longer batches into
// consecutive launches, which preserves array order.
#pragma once
#include "k_select.h"
#include "layout.h"

namespace evk {

constexpr int UPD_CHUNK = 8192;

__global__ __launch_bounds__(1024) void k_update_q(const int32_t* __restrict__ ids, const float* __restrict__ rewards,
                                                   int M, float* __restrict__ qstage, int64_t N, float alpha,
                                                   uint32_t* __restrict__ counters) {
    __shared__ uint64_t keys[UPD_CHUNK];     // (id << 32 | position) while sorting, then (id, reward)
    const int tid = threadIdx.x;
    int npad = 2;
    while (npad < M) npad <<= 1;
    uint32_t bad = 0;
    for (int i = tid; i < npad; i += 1024) {
        uint64_t k = ~0ull;                  // padding and invalid ids sort to the end
        if (i < M) {
            int32_t id = ids[i];
            if (id >= 0 && (int64_t)id < N) k = ((uint64_t)(uint32_t)id << 32) | (uint32_t)i;
            else ++bad;
        }
        keys[i] = k;
    }
    if (bad) atomicAdd(counters, bad);       // integer diagnostic counter, not a Q value
    __syncthreads();
    // ascending sort = descending with the comparison reversed
    bitonic_desc(keys, npad, tid, 1024, [](uint64_t x, uint64_t y) { return x > y; });
    // replace positions by the rewards they point to
    for (int i = tid; i < npad; i += 1024) {
        uint64_t k = keys[i];
        if (k != ~0ull) {
            float r = rewards[(uint32_t)k];
            keys[i] = (k & 0xffffffff00000000ull) | __float_as_uint(r);
        }
    }
    __syncthreads();
    for (int i = tid; i < npad; i += 1024) {
        uint64_t k = keys[i];
        if (k == ~0ull) continue;
        uint32_t id = (uint32_t)(k >> 32);
        if (i > 0 && (uint32_t)(keys[i - 1] >> 32) == id) continue;   // not the head of its segment
        float q = qstage[id];
        int j = i;
        do {
#pragma clang fp contract(off)   // three separately rounded operations, never a fused multiply-add
            float r = __uint_as_float((uint32_t)keys[j]);
            float diff = r - q;
            float stepv = alpha * diff;
            q = q + stepv;
            ++j;
        } while (j < npad && (uint32_t)(keys[j] >> 32) == id && keys[j] != ~0ull);
        qstage[id] = q;
    }
}

}  // namespace evk
