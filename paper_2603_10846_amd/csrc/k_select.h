// Selection kernels: survivor lists -> candidate pool -> value filter (Sec. 3.2).
#pragma once
#include "k_ingest.h"
#include "layout.h"

namespace evk {

// In-LDS bitonic sort, descending, n a power of two, all threads of the workgroup take part.
template <typename T, typename Less>
__device__ __forceinline__ void bitonic_desc(T* a, int n, int tid, int nthreads, Less less) {
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int p = tid; p < (n >> 1); p += nthreads) {
                int i = ((p & ~(j - 1)) << 1) | (p & (j - 1));   // index with bit j clear
                int l = i | j;
                bool desc = (i & k) == 0;
                T x = a[i], y = a[l];
                if (less(x, y) == desc) { a[i] = y; a[l] = x; }
            }
            __syncthreads();
        }
}

// After a scan pass, for one query: find the k1-th best survivor key (similarity desc, id asc) by
// an MSB-first radix select over the packed 64-bit keys, set the next pass's threshold to that
// similarity minus `margin` (a bound on the scan's fp32 rounding error, so that no true member of
// the pool can be filtered out; pre-divided by the query's inverse norm because the scan compares
// before applying it), and compact every key whose similarity reaches that threshold to the head of
// the list: these seed the next pass and, after the last pass, are the candidates that get re-scored
// in fp64.  Nothing is sorted here -- slot order is irrelevant to every consumer.
// Keys live in registers (8 per lane, 1024 lanes); each radix pass builds per-wavefront digit
// histograms in LDS, sums them, and one wavefront picks the digit by a suffix scan.
__global__ __launch_bounds__(1024) void k_select(uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt,
                                                 float* __restrict__ thr, const float* __restrict__ invq,
                                                 uint32_t* __restrict__ counters, int k1, float margin) {
    __shared__ uint32_t hist[16][256];
    __shared__ uint32_t tot[256];
    __shared__ uint64_t pivot_s;
    __shared__ uint32_t sel_digit, sel_need, sel_single, band_s, nout_s;
    const int b = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    uint64_t* list = surv + (int64_t)b * SURV_CAP;
    const uint32_t raw = cnt[b];
    const int n = raw > (uint32_t)SURV_CAP ? SURV_CAP : (int)raw;
    if (raw > (uint32_t)SURV_CAP && tid == 0) atomicAdd(counters + 1, 1u);
    if (n < k1) {                       // fewer rows than the pool size: keep them all, no threshold
        if (tid == 0) { cnt[b] = (uint32_t)n; thr[b] = -2.0f / invq[b]; }   // finite floor, see k_prep_queries
        return;
    }
    uint64_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { int idx = i * 1024 + tid; key[i] = idx < n ? list[idx] : 0ull; }   // 0 = empty
    if (tid == 0) { band_s = 0; nout_s = 0; }
    uint64_t prefix = 0, pivot = 0;
    uint32_t need = (uint32_t)k1;
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        for (int i = tid; i < 16 * 256; i += 1024) (&hist[0][0])[i] = 0;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (key[i] != 0 && (pass == 0 || (key[i] >> (shift + 8)) == (prefix >> (shift + 8))))
                atomicAdd(&hist[wave][(uint32_t)(key[i] >> shift) & 255u], 1u);
        __syncthreads();
        if (tid < 256) {
            uint32_t s = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) s += hist[w][tid];
            tot[tid] = s;
        }
        __syncthreads();
        if (wave == 0) {                // lane l owns digits 4l .. 4l+3; larger digit = better key
            uint32_t c[4] = {tot[4 * lane], tot[4 * lane + 1], tot[4 * lane + 2], tot[4 * lane + 3]};
            uint32_t local = c[0] + c[1] + c[2] + c[3], incl = local;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) { uint32_t t = __shfl_down(incl, o, 64); if (lane + o < 64) incl += t; }
            uint32_t run = incl - local;            // keys with a digit in a higher lane
#pragma unroll
            for (int k = 3; k >= 0; --k) {
                if (run < need && run + c[k] >= need) { sel_digit = 4 * lane + k; sel_need = need - run; sel_single = c[k] == 1; }
                run += c[k];
            }
        }
        __syncthreads();
        prefix |= (uint64_t)sel_digit << shift;
        need = sel_need;
        if (sel_single || pass == 7) {              // one key left under this prefix: it is the k1-th best
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (key[i] != 0 && (key[i] >> shift) == (prefix >> shift)) pivot_s = key[i];
            __syncthreads();
            pivot = pivot_s;
            break;
        }
    }
    const float tau = key_sim(pivot) - margin;
    uint64_t cutkey = (uint64_t)f2ord(tau) << 32;   // every key with similarity >= tau compares >= cutkey
    uint32_t mine = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) mine += key[i] != 0 && key[i] >= cutkey;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) mine += __shfl_xor(mine, o, 64);
    if (lane == 0 && mine) atomicAdd(&band_s, mine);
    __syncthreads();
    if (band_s > (uint32_t)KEEP_MAX) cutkey = pivot;    // band too crowded: keep exactly the k1 best
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (key[i] != 0 && key[i] >= cutkey) list[atomicAdd(&nout_s, 1u)] = key[i];
    __syncthreads();
    if (tid == 0) { cnt[b] = nout_s; thr[b] = tau / invq[b]; }
}

// Exact similarities of the selected candidates: one wavefront per (query, candidate) re-reads the
// stored row and accumulates dot product and squared norm in fp64 (products of 16-bit values are
// exact, so this is the cosine of the stored vectors up to fp64 rounding).
template <int DT>
__global__ __launch_bounds__(256) void k_rescore(const void* __restrict__ store_, const float* __restrict__ qf,
                                                 const double* __restrict__ invq64, const uint64_t* __restrict__ surv,
                                                 const uint32_t* __restrict__ cnt, double* __restrict__ exact,
                                                 int nkb) {
    const int b = blockIdx.y, lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (j >= (int)cnt[b]) return;
    const int32_t id = key_id(surv[(int64_t)b * SURV_CAP + j]);
    const float* q = qf + (int64_t)b * nkb * KB;
    double dot = 0.0, ssq = 0.0;
    if (DT == 0) {
        const float* store = static_cast<const float*>(store_);
        for (int c4 = lane; c4 < nkb * 16; c4 += 64) {
            float4 x = *reinterpret_cast<const float4*>(store + off32(id, c4, nkb));
            float4 y = *reinterpret_cast<const float4*>(q + c4 * 4);
            dot += (double)x.x * y.x + (double)x.y * y.y + (double)x.z * y.z + (double)x.w * y.w;
            ssq += (double)x.x * x.x + (double)x.y * x.y + (double)x.z * x.z + (double)x.w * x.w;
        }
    } else {
        const uint16_t* store = static_cast<const uint16_t*>(store_);
        for (int c8 = lane; c8 < nkb * 8; c8 += 64) {
            uint4 pk = *reinterpret_cast<const uint4*>(store + off16(id, c8, nkb));
            uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                uint16_t lo = (uint16_t)(w[i] & 0xffff), hi = (uint16_t)(w[i] >> 16);
                double x0 = DT == 1 ? bf16_to_f(lo) : f16_to_f(lo);
                double x1 = DT == 1 ? bf16_to_f(hi) : f16_to_f(hi);
                dot += x0 * (double)q[c8 * 8 + 2 * i] + x1 * (double)q[c8 * 8 + 2 * i + 1];
                ssq += x0 * x0 + x1 * x1;
            }
        }
    }
    dot = wave_sum_d(dot);
    ssq = wave_sum_d(ssq);
    if (lane == 0) exact[(int64_t)b * KEEP_MAX + j] = dot * invq64[b] * (1.0 / sqrt(ssq));
}

struct SimId { double v; int32_t id; };
__device__ __forceinline__ bool simid_less(const SimId& x, const SimId& y) {   // "x ranks below y"
    return x.v < y.v || (x.v == y.v && x.id > y.id);
}

// Deterministic sum of f(j), j < n, over a 256-thread workgroup (fixed tree).
template <typename F>
__device__ __forceinline__ double block_sum(double* red, int tid, int n, F f) {
    double s = 0.0;
    for (int j = tid; j < n; j += 256) s += f(j);
    red[tid] = s;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) { if (tid < st) red[tid] += red[tid + st]; __syncthreads(); }
    double r = red[0];
    __syncthreads();
    return r;
}

// Candidate pool and value filter for one query (Sec. 3.2): order the re-scored candidates by
// (similarity desc, id asc), keep k1 as the pool C(x); gather the stage's Q values; z-score both
// over the pool (population deviation, denominator std + 1e-6); score = (1-lambda) z_s + lambda z_q;
// emit the k2 best by (score desc, id asc).  All in fp64, scores rounded to fp32 on output.
__global__ __launch_bounds__(256) void k_rerank(const uint64_t* __restrict__ surv, const uint32_t* __restrict__ cnt,
                                                const double* __restrict__ exact, const float* __restrict__ qstage,
                                                int k1, int k2, double lambda, int32_t* __restrict__ out_ids,
                                                float* __restrict__ out_scores, int32_t* __restrict__ cand_ids,
                                                float* __restrict__ cand_sims) {
    __shared__ SimId a[KEEP_MAX];
    __shared__ double qv[MEM_MAX_K1_INTERNAL];
    __shared__ double red[256];
    const int b = blockIdx.x, tid = threadIdx.x;
    const int kk = (int)cnt[b];
    for (int i = tid; i < KEEP_MAX; i += 256) {
        SimId e;
        if (i < kk) { e.v = exact[(int64_t)b * KEEP_MAX + i]; e.id = key_id(surv[(int64_t)b * SURV_CAP + i]); }
        else        { e.v = -INFINITY; e.id = 0x7fffffff; }
        a[i] = e;
    }
    __syncthreads();
    bitonic_desc(a, KEEP_MAX, tid, 256, simid_less);
    const int k1e = kk < k1 ? kk : k1;
    if (cand_ids)
        for (int i = tid; i < k1; i += 256) {
            cand_ids[(int64_t)b * k1 + i] = i < k1e ? a[i].id : -1;
            cand_sims[(int64_t)b * k1 + i] = i < k1e ? (float)a[i].v : -INFINITY;
        }
    for (int i = tid; i < k1e; i += 256) qv[i] = (double)qstage[a[i].id];
    __syncthreads();
    double scale_s = 0.0, scale_q = 0.0, mean_s = 0.0, mean_q = 0.0;
    if (k1e > 0) {
        mean_s = block_sum(red, tid, k1e, [&](int j) { return a[j].v; }) / k1e;
        mean_q = block_sum(red, tid, k1e, [&](int j) { return qv[j]; }) / k1e;
        double var_s = block_sum(red, tid, k1e, [&](int j) { double x = a[j].v - mean_s; return x * x; }) / k1e;
        double var_q = block_sum(red, tid, k1e, [&](int j) { double x = qv[j] - mean_q; return x * x; }) / k1e;
        scale_s = 1.0 / (sqrt(var_s) + 1e-6);
        scale_q = 1.0 / (sqrt(var_q) + 1e-6);
    }
    // scores overwrite the similarities of the pool; the rest of the array becomes padding
    for (int i = tid; i < KEEP_MAX; i += 256) {
        SimId e = a[i];
        if (i < k1e) e.v = (1.0 - lambda) * ((e.v - mean_s) * scale_s) + lambda * ((qv[i] - mean_q) * scale_q);
        else { e.v = -INFINITY; e.id = 0x7fffffff; }
        a[i] = e;
    }
    __syncthreads();
    bitonic_desc(a, MEM_MAX_K1_INTERNAL, tid, 256, simid_less);
    const int k2e = k1e < k2 ? k1e : k2;
    for (int i = tid; i < k2; i += 256) {
        out_ids[(int64_t)b * k2 + i] = i < k2e ? a[i].id : -1;
        out_scores[(int64_t)b * k2 + i] = i < k2e ? (float)a[i].v : -INFINITY;
    }
}

}  // namespace evk
