// Start-point selection (Sec. 3.4, continual refining): out of a task's set P(x) of optimisation
// start points, the one with the largest value in the stage's Q table (lower id among equals, a NaN
// value counting as -inf), or -- epsilon-greedy, the policy Sec. 4.4 states for start points as for
// contexts -- with probability eps the member at a uniformly random position of the set.
//
// One workgroup per set; the G sets of a call are one id array and G + 1 offsets.  A set is a few
// to a few hundred ids and each costs one gathered 4-byte value, so the kernel is a latency-bound
// gather: every lane requests its ids' values at once, the maximum is a wavefront butterfly on a
// 64-bit key, and only an exploring set walks its ids a second time (to find the drawn position
// among the members, ids outside the bank not being members).
#pragma once
#include "k_select.h"
#include "layout.h"

namespace evk {

constexpr int SP_LANES = 256;

// Order-preserving key of (value desc, id asc): larger key = better.  -0 and +0 must tie, so zero
// is canonicalised first; NaN ranks with -inf.
__device__ __forceinline__ uint64_t startpoint_key(float q, int32_t id) {
    if (q != q) q = -INFINITY;
    if (q == 0.f) q = 0.f;                                   // -0 -> +0
    uint32_t u = __float_as_uint(q);
    u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);          // monotone in the value
    return ((uint64_t)u << 32) | (uint32_t)(0x7fffffff - id);
}

__device__ __forceinline__ uint64_t wave_max_u64(uint64_t x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        const uint64_t y = __shfl_xor(x, m);
        x = y > x ? y : x;
    }
    return x;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t x) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x += (uint32_t)__shfl_xor((int)x, m);
    return x;
}

__global__ __launch_bounds__(SP_LANES) void k_select_by_q(const int32_t* __restrict__ set_ids, int64_t n_ids,
                                                          const int64_t* __restrict__ set_offsets,
                                                          const float* __restrict__ qstage, int64_t N, EpsGreedy eg,
                                                          int32_t* __restrict__ out_id, float* __restrict__ out_q,
                                                          uint32_t* __restrict__ counters) {
    __shared__ uint64_t best_s[SP_LANES / 64];
    __shared__ uint32_t members_s[SP_LANES / 64], bad_s[SP_LANES / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t g = blockIdx.x;
    // offsets are clamped to the id array, so a malformed offset table cannot cause a read outside it
    auto clamped = [&](int64_t o) { return o < 0 ? (int64_t)0 : o > n_ids ? n_ids : o; };
    const int64_t first = clamped(set_offsets[g]), last = clamped(set_offsets[g + 1]);

    // greedy pass: best key, number of members, number of ids that are none
    uint64_t best = 0;                                       // below every real key (a key has bit 63 or its complement set)
    uint32_t members = 0, bad = 0;
    for (int64_t i0 = first + tid; i0 < last; i0 += 4 * SP_LANES) {
        int32_t id[4];
        float q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + u * SP_LANES;
            id[u] = i < last ? set_ids[i] : -1;
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) q[u] = (id[u] >= 0 && (int64_t)id[u] < N) ? qstage[id[u]] : 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int64_t i = i0 + u * SP_LANES;
            if (i >= last) continue;
            if (id[u] >= 0 && (int64_t)id[u] < N) {
                const uint64_t k = startpoint_key(q[u], id[u]);
                best = k > best ? k : best;
                ++members;
            } else {
                ++bad;
            }
        }
    }
    best = wave_max_u64(best);
    members = wave_sum_u32(members);
    bad = wave_sum_u32(bad);
    if (lane == 0) { best_s[wave] = best; members_s[wave] = members; bad_s[wave] = bad; }
    __syncthreads();
    best = 0; members = 0; bad = 0;
#pragma unroll
    for (int w = 0; w < SP_LANES / 64; ++w) {
        best = best_s[w] > best ? best_s[w] : best;
        members += members_s[w];
        bad += bad_s[w];
    }
    if (tid == 0 && bad) atomicAdd(counters, bad);           // integer diagnostic counter
    if (members == 0) {
        if (tid == 0) {
            out_id[g] = -1;
            out_q[g] = 0.f;
            if (eg.explored) eg.explored[g] = 0;
        }
        return;
    }
    // the set's draw: every lane computes the same words
    const philox_out r = philox4x32_10((uint32_t)eg.step, (uint32_t)(eg.step >> 32), g, 0xffffffffu,
                                       (uint32_t)eg.seed, (uint32_t)(eg.seed >> 32));
    const bool explore = (uint64_t)r.w0 < eg.threshold;
    if (!explore) {
        if (tid == 0) {
            const int32_t id = 0x7fffffff - (int32_t)(uint32_t)best;
            out_id[g] = id;
            out_q[g] = qstage[id];
            if (eg.explored) eg.explored[g] = 0;
        }
        return;
    }
    // exploring: the member at position `want` among the members in array order
    const uint32_t want = (uint32_t)(((uint64_t)r.w1 * members) >> 32);
    __shared__ uint32_t chunk_s[SP_LANES / 64];
    uint32_t before = 0;                                     // members in earlier chunks (uniform)
    for (int64_t i0 = first; i0 < last; i0 += SP_LANES) {
        const int64_t i = i0 + tid;
        const int32_t id = i < last ? set_ids[i] : -1;
        const bool is_member = id >= 0 && (int64_t)id < N;
        const uint64_t ballot = __builtin_amdgcn_ballot_w64(is_member);
        if (lane == 0) chunk_s[wave] = (uint32_t)__popcll(ballot);
        __syncthreads();
        uint32_t mine = before, total = 0;
#pragma unroll
        for (int w = 0; w < SP_LANES / 64; ++w) {
            if (w < wave) mine += chunk_s[w];
            total += chunk_s[w];
        }
        mine += (uint32_t)__popcll(ballot & ((1ull << lane) - 1ull));
        if (is_member && mine == want) {
            out_id[g] = id;
            out_q[g] = qstage[id];
            if (eg.explored) eg.explored[g] = 1;
        }
        before += total;
        if (before > want) break;                            // uniform: found
        __syncthreads();
    }
}

}  // namespace evk
