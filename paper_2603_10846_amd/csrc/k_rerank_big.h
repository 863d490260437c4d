// Candidate pool and value filter for pools of more than 256 candidates (up to 2048): the pool-size
// study of Sec. 4.4 over-retrieves by a multiple of the final context size.  Same computation as
// k_rerank (Sec. 3.2): order the re-scored candidates by (similarity desc, id asc), keep k1 as the
// pool, gather the stage's Q values, z-score both over the pool (population deviation, denominator
// std + 1e-6), score = (1-lambda) z_s + lambda z_q, emit the k2 best by (score desc, id asc) -- or
// fill the k2 slots epsilon-greedily (Sec. 3.3).  All in fp64.
// With thousands of entries counting ranks is quadratic work, so both orderings are bitonic sorts of
// an index array in LDS (1024 lanes); sums for the z-scores are taken per lane over a fixed stride,
// then per wavefront, then over the 16 wavefront partials in a fixed order.
#pragma once
#include "k_select.h"

namespace evk {

constexpr int BIG_T = 1024;

// LDS (dynamic), in this order: val[cap] f64, sco[k1p] f64, red[16] f64, taken[k1p / 64] u64, kid[cap] i32,
// idx[cap] u32, pid[k1p] i32, word0[k2p] u32, word1[k2p] u32; cap = the padded list length (a power of two
// >= the number of candidates), k1p / k2p = k1 / k2 rounded up to a multiple of 64.
__host__ __device__ __forceinline__ int pad64(int x) { return (x + 63) & ~63; }
__host__ __device__ __forceinline__ size_t rerank_big_lds(int cap, int k1, int k2) {
    return (size_t)cap * 16 + (size_t)pad64(k1) * 12 + 16 * 8 + (size_t)pad64(k1) / 8 + (size_t)pad64(k2) * 8;
}

__device__ __forceinline__ double block_sum_big(double* red, int tid, double x) {
    x = wave_sum_d(x);
    if ((tid & 63) == 0) red[tid >> 6] = x;
    __syncthreads();
    double r = 0.0;
#pragma unroll
    for (int w = 0; w < 16; ++w) r += red[w];
    __syncthreads();
    return r;
}

__global__ __launch_bounds__(BIG_T) void k_rerank_big(const uint64_t* __restrict__ surv, const uint32_t* __restrict__ cnt,
                                                     const double* __restrict__ exact, int exact_stride,
                                                     const float* __restrict__ qstage, int k1, int k2, double lambda,
                                                     int cap, int32_t* __restrict__ out_ids, float* __restrict__ out_scores,
                                                     int32_t* __restrict__ cand_ids, float* __restrict__ cand_sims,
                                                     EpsGreedy eg) {
    extern __shared__ __align__(16) unsigned char big_smem[];
    const int k1p = pad64(k1), k2p = pad64(k2);
    double* val = reinterpret_cast<double*>(big_smem);
    double* sco = val + cap;
    double* red = sco + k1p;
    uint64_t* taken = reinterpret_cast<uint64_t*>(red + 16);
    int32_t* kid = reinterpret_cast<int32_t*>(taken + k1p / 64);
    uint32_t* idx = reinterpret_cast<uint32_t*>(kid + cap);
    int32_t* pid = reinterpret_cast<int32_t*>(idx + cap);
    uint32_t* word0 = reinterpret_cast<uint32_t*>(pid + k1p);
    uint32_t* word1 = word0 + k2p;
    const int b = blockIdx.x, tid = threadIdx.x;
    const int kk = (int)cnt[b];
    for (int i = tid; i < cap; i += BIG_T) {
        const bool live = i < kk;
        val[i] = live ? finite_or_lowest(exact[(int64_t)b * exact_stride + i]) : -INFINITY;     // padding sorts last (its id is the largest)
        kid[i] = live ? key_id(surv[(int64_t)b * SURV_CAP + i]) : 0x7fffffff;
        idx[i] = (uint32_t)i;
    }
    __syncthreads();
    const int k1e = kk < k1 ? kk : k1;
    // ordering 1: indices by (similarity desc, id asc)
    bitonic_desc(idx, cap, tid, BIG_T, [&](uint32_t x, uint32_t y) { return ranks_before(val[y], kid[y], val[x], kid[x]); });
    for (int i = tid; i < k1; i += BIG_T) {
        const bool live = i < k1e;
        const uint32_t s = idx[i];
        if (cand_ids) {
            cand_ids[(int64_t)b * k1 + i] = live ? kid[s] : -1;
            cand_sims[(int64_t)b * k1 + i] = live ? (float)val[s] : -INFINITY;
        }
        if (live) { sco[i] = val[s]; pid[i] = kid[s]; }
    }
    __syncthreads();
    // z-scores over the pool: pool entry i belongs to lane i % 1024
    double sim[2], qv[2];
    double s_sim = 0.0, s_q = 0.0;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int i = tid + u * BIG_T;
        const bool mine = i < k1e;
        sim[u] = mine ? sco[i] : 0.0;
        qv[u] = mine ? (double)qstage[pid[i]] : 0.0;
        s_sim += sim[u];
        s_q += qv[u];
    }
    if (k1e > 0) {                                                    // uniform
        const double mean_s = block_sum_big(red, tid, s_sim) / k1e;
        const double mean_q = block_sum_big(red, tid, s_q) / k1e;
        double d_s[2], d_q[2], v_s = 0.0, v_q = 0.0;
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const bool mine = tid + u * BIG_T < k1e;
            d_s[u] = mine ? sim[u] - mean_s : 0.0;
            d_q[u] = mine ? qv[u] - mean_q : 0.0;
            v_s += d_s[u] * d_s[u];
            v_q += d_q[u] * d_q[u];
        }
        const double var_s = block_sum_big(red, tid, v_s) / k1e;
        const double var_q = block_sum_big(red, tid, v_q) / k1e;
        const double scale_s = 1.0 / (sqrt(var_s) + 1e-6), scale_q = 1.0 / (sqrt(var_q) + 1e-6);
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = tid + u * BIG_T;
            if (i < k1e) sco[i] = finite_or_lowest((1.0 - lambda) * (d_s[u] * scale_s) + lambda * (d_q[u] * scale_q));
        }
    }
    // ordering 2: pool positions by (score desc, id asc); the index array is reused (pool padded to a power of two)
    int cap2 = 2;
    while (cap2 < k1e) cap2 <<= 1;
    __syncthreads();
    for (int i = tid; i < cap2; i += BIG_T) idx[i] = (uint32_t)i;
    __syncthreads();
    bitonic_desc(idx, cap2, tid, BIG_T, [&](uint32_t x, uint32_t y) {
        const bool lx = (int)x < k1e, ly = (int)y < k1e;                   // padding positions sort last
        if (!lx || !ly) return !lx && ly;
        return ranks_before(sco[y], pid[y], sco[x], pid[x]);
    });
    const int k2e = k1e < k2 ? k1e : k2;
    const bool greedy = eg.threshold == 0 && eg.explored == nullptr;
    for (int j = tid; j < k2; j += BIG_T) {
        const bool live = j < k2e;
        if (greedy || !live) {
            out_ids[(int64_t)b * k2 + j] = live ? pid[idx[j]] : -1;
            out_scores[(int64_t)b * k2 + j] = live ? (float)sco[idx[j]] : -INFINITY;
            if (eg.explored) eg.explored[(int64_t)b * k2 + j] = 0;
        }
    }
    if (greedy) return;                                               // uniform
    // Epsilon-greedy slot filling (Sec. 3.3): draws per slot in parallel, then one lane fills the slots in
    // order from an occupancy bit mask over the greedy order (kept in LDS: up to 2048 bits).
    __syncthreads();
    for (int j = tid; j < k2e; j += BIG_T) {
        const philox_out r = philox4x32_10((uint32_t)eg.step, (uint32_t)(eg.step >> 32), (uint32_t)b, (uint32_t)j,
                                           (uint32_t)eg.seed, (uint32_t)(eg.seed >> 32));
        word0[j] = r.w0;
        word1[j] = r.w1;
    }
    const int nwords = (k1e + 63) / 64;
    for (int w = tid; w < nwords; w += BIG_T) {
        const int lo = w * 64;
        taken[w] = k1e >= lo + 64 ? 0ull : (~0ull << (k1e - lo));
    }
    __syncthreads();
    if (tid == 0) {
        for (int j = 0; j < k2e; ++j) {
            const bool explore = (uint64_t)word0[j] < eg.threshold;
            int want = explore ? (int)(((uint64_t)word1[j] * (uint32_t)(k1e - j)) >> 32) : 0;   // index among the free members
            int pos = 0;
            for (int w = 0; w < nwords; ++w) {
                uint64_t fr = ~taken[w];
                const int c = __popcll(fr);
                if (want < c) {
                    for (int t = 0; t < want; ++t) fr &= fr - 1;              // drop the `want` lowest free bits
                    const int bit = __ffsll((long long)fr) - 1;
                    taken[w] |= 1ull << bit;
                    pos = w * 64 + bit;
                    break;
                }
                want -= c;
            }
            out_ids[(int64_t)b * k2 + j] = pid[idx[pos]];
            out_scores[(int64_t)b * k2 + j] = (float)sco[idx[pos]];
            if (eg.explored) eg.explored[(int64_t)b * k2 + j] = explore ? 1 : 0;
        }
    }
}

}  // namespace evk
