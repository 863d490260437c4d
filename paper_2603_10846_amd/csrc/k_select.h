// Selection kernels: survivor lists -> candidate pool -> value filter (Sec. 3.2).
#pragma once
#include <type_traits>

#include "k_ingest.h"
#include "layout.h"

namespace evk {

// In-LDS bitonic sort, descending, n a power of two, all threads of the workgroup take part.
// Pair p of a stage belongs to thread p % nthreads, so a wavefront always works on the same
// 128-element blocks; a stage with stride j <= 64 stays inside those blocks.  Hence a workgroup
// barrier is needed only next to a stage with a larger stride -- between two small-stride stages
// (and always in a one-wavefront workgroup) the wavefront's own in-order LDS accesses suffice.
template <typename T, typename Less>
__device__ __forceinline__ void bitonic_desc(T* a, int n, int tid, int nthreads, Less less) {
    int prev_j = 1 << 30;                                     // "large": the caller's writes came from any thread
    for (int k = 2; k <= n; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            if (nthreads > 64 && (j > 64 || prev_j > 64)) __syncthreads();
            else __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
            for (int p = tid; p < (n >> 1); p += nthreads) {
                int i = ((p & ~(j - 1)) << 1) | (p & (j - 1));   // index with bit j clear
                int l = i | j;
                bool desc = (i & k) == 0;
                T x = a[i], y = a[l];
                if (less(x, y) == desc) { a[i] = y; a[l] = x; }
            }
            prev_j = j;
        }
    __syncthreads();
}

// OR over the 64 lanes of a wavefront (all lanes active); lane 63 ends up with the result.
__device__ __forceinline__ uint32_t wave_or_u32(uint32_t x) {
    int v = (int)x;
    v |= __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v |= __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v |= __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v |= __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v |= __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true);   // row_bcast:15 into rows 1 and 3
    v |= __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true);   // row_bcast:31 into rows 2 and 3
    return (uint32_t)v;
}

// After a scan pass, for one query: find the k1-th best survivor key (similarity desc, id asc) by
// an MSB-first radix select over the packed 64-bit keys, set the next pass's threshold to that
// similarity minus `margin` (a bound on the scan's fp32 rounding error, so that no true member of
// the pool can be filtered out; pre-divided by the query's inverse norm because the scan compares
// before applying it), and compact every key whose similarity reaches that threshold to the head of
// the list: these seed the next pass and, after the last pass, are the candidates that get re-scored
// in fp64.  Nothing is sorted here -- slot order is irrelevant to every consumer.
// Keys live in registers (8 per lane, 1024 lanes); the passes start at the highest bit on which two
// keys differ; each builds per-wavefront digit histograms in LDS, sums them, and one wavefront
// picks the digit by a suffix scan.
// A list that overflowed during the pass (more than SURV_CAP rows reached the threshold; the surplus was
// dropped) is counted and the query is flagged: its pool may then miss members.
// More than keep_max keys inside the margin ("crowded band"; near-duplicate entries do that):
//   SEL_PASS   (between scan passes) every key of the band is kept -- any of them may belong to the pool;
//   SEL_FINAL  (after the last pass) likewise, and the function returns true: the caller replaces the
//              keys' similarities by exactly accumulated ones (rescore_one_query<DT, true>) and selects
//              again with a margin of two fp32 roundings;
//   SEL_EXACT  (that second selection) a band that is still crowded can only be one of ties within
//              fp32 resolution: the k1 best keys are kept, lower ids first among equal similarities.
enum { SEL_PASS = 0, SEL_FINAL = 1, SEL_EXACT = 2 };
__device__ __forceinline__ bool select_one_query(const int b, uint64_t* surv, uint32_t* cnt,
                                                 float* thr, const float* invq, uint32_t* counters, uint32_t* flags,
                                                 int k1, float margin, int may_have_empty, int keep_max, int mode) {
    __shared__ uint32_t hist[16][256];
    __shared__ uint32_t tot[256];
    __shared__ uint64_t pivot_s, or_s[16];
    __shared__ uint32_t sel_digit, sel_need, sel_single, band_s, nout_s;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    uint64_t* list = surv + (int64_t)b * SURV_CAP;
    const uint32_t raw = cnt[b];
    const int n = raw > (uint32_t)SURV_CAP ? SURV_CAP : (int)raw;
    if (raw > (uint32_t)SURV_CAP && tid == 0) { atomicAdd(counters + 1, 1u); flags[b] |= 1u; }
    if (!may_have_empty && n < k1) {    // fewer rows than the pool size: keep them all, no threshold
        if (tid == 0) { cnt[b] = (uint32_t)n; thr[b] = -2.0f / invq[b]; }   // finite floor, see k_prep_queries
        return false;
    }
    uint64_t key[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) { int idx = i * 1024 + tid; key[i] = idx < n ? list[idx] : 0ull; }   // 0 = empty
    const uint64_t ref = n > 0 ? list[0] : 0ull;      // any one key (or an empty slot), see the radix passes
    if (tid == 0) { band_s = 0; nout_s = 0; }
    if (may_have_empty) {               // uniform
        // A masked sparsest pass leaves the slots of rows the query does not accept empty (key 0): if
        // fewer than k1 slots are in use, keep those (compacted to the head of the list), no threshold.
        uint32_t used = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) used += key[i] != 0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) used += __shfl_xor(used, o, 64);
        __syncthreads();
        if (lane == 0 && used) atomicAdd(&band_s, used);
        __syncthreads();
        if (band_s < (uint32_t)k1) {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (key[i] != 0) list[atomicAdd(&nout_s, 1u)] = key[i];
            __syncthreads();
            if (tid == 0) { cnt[b] = nout_s; thr[b] = -2.0f / invq[b]; }
            return false;
        }
        __syncthreads();
        if (tid == 0) band_s = 0;
        __syncthreads();
    }
    // Bits that all keys share need no pass: the survivors of a filtering pass lie in a narrow band
    // of similarities, so the leading 12-20 bits of their keys are the same, and a pass over such
    // bits would also send every key to one histogram bin (same-address LDS atomics serialise).
    // (the bits on which some key differs from the list's first key, OR-ed over the workgroup)
    uint64_t differ = 0ull;
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (key[i] != 0) differ |= key[i] ^ ref;
    differ = ((uint64_t)wave_or_u32((uint32_t)(differ >> 32)) << 32) | wave_or_u32((uint32_t)differ);
    if (lane == 63) or_s[wave] = differ;
    for (int i = tid; i < 16 * 256; i += 1024) (&hist[0][0])[i] = 0;
    __syncthreads();
    differ = 0ull;
#pragma unroll
    for (int w = 0; w < 16; ++w) differ |= or_s[w];               // 0 only if there is a single key
    int hi = differ ? 63 - __builtin_clzll(differ) : 7;           // highest bit on which two keys differ
    uint64_t prefix = hi < 63 ? (ref >> (hi + 1)) << (hi + 1) : 0ull, pivot = 0;
    uint32_t need = (uint32_t)k1;
    for (;;) {
        const int shift = hi >= 7 ? hi - 7 : 0;               // this pass ranks bits hi .. shift
        const uint32_t dmask = (1u << (hi - shift + 1)) - 1u;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (key[i] != 0 && (hi == 63 || (key[i] >> (hi + 1)) == (prefix >> (hi + 1))))
                atomicAdd(&hist[wave][(uint32_t)(key[i] >> shift) & dmask], 1u);
        __syncthreads();
        if (tid < 256) {
            uint32_t sum = 0;
#pragma unroll
            for (int w = 0; w < 16; ++w) { sum += hist[w][tid]; hist[w][tid] = 0; }   // cleared for the next pass
            tot[tid] = sum;
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
        if (sel_single || shift == 0) {             // one key left under this prefix: it is the k1-th best
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (key[i] != 0 && (key[i] >> shift) == (prefix >> shift)) pivot_s = key[i];
            __syncthreads();
            pivot = pivot_s;
            break;
        }
        hi = shift - 1;
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
    const bool crowded = band_s > (uint32_t)keep_max;   // uniform
    if (crowded && mode == SEL_EXACT) cutkey = pivot;   // ties within fp32 resolution: exactly the k1 best
#pragma unroll
    for (int i = 0; i < 8; ++i)
        if (key[i] != 0 && key[i] >= cutkey) list[atomicAdd(&nout_s, 1u)] = key[i];
    __syncthreads();
    if (tid == 0) { cnt[b] = nout_s; thr[b] = tau / invq[b]; }
    return crowded && mode == SEL_FINAL;
}

__global__ __launch_bounds__(1024) void k_select(uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt,
                                                 float* __restrict__ thr, const float* __restrict__ invq,
                                                 uint32_t* __restrict__ counters, uint32_t* __restrict__ flags, int k1, float margin,
                                                 int may_have_empty, int keep_max) {
    select_one_query((int)blockIdx.x, surv, cnt, thr, invq, counters, flags, k1, margin, may_have_empty, keep_max, SEL_PASS);
}

// Exact similarities of the selected candidates: one wavefront per (query, candidate) re-reads the
// stored row and accumulates dot product and squared norm in fp64 (products of 16-bit values are
// exact, so this is the cosine of the stored vectors up to fp64 rounding).
// REQUANT: instead of storing the fp64 similarity, the candidate's key is rewritten with it (rounded to
// fp32: resolution 6e-8), for a second selection over a crowded band.
template <int DT, bool REQUANT = false>
__device__ __forceinline__ void rescore_one_query(const int b, const int part, const int parts,
                                                  const void* store_, const float* qf,
                                                  const double* invq64, std::conditional_t<REQUANT, uint64_t, const uint64_t>* surv,
                                                  const uint32_t* cnt, double* exact,
                                                  int nkb, int exact_stride, int begin = 0) {
    // One workgroup per query; 16 lanes per candidate row, so a wavefront works on four rows at a
    // time and every lane has up to eight 16-byte loads in flight.
    const int sub = threadIdx.x & 15, grp = threadIdx.x >> 4;   // grp 0..63
    const int n = (int)cnt[b];
    const float* q = qf + (int64_t)b * nkb * KB;
    constexpr int EPC = DT == 0 ? 4 : 8;                 // elements per 16-byte chunk
    const int nch = nkb * KB / EPC;                      // chunks per row
    // (`parts` workgroups share a query: workgroup `part` takes the candidate groups part, part + parts, ...)
    for (int j0 = begin + 64 * part; j0 < n; j0 += 64 * parts) {   // uniform trip count: the shuffles below need all lanes
        const int j = j0 + grp;
        const bool live = j < n;
        const int32_t id = live ? key_id(surv[(int64_t)b * SURV_CAP + j]) : 0;
        double dot = 0.0, ssq = 0.0;
        for (int c0 = sub; c0 < nch; c0 += 16 * 8) {
            uint4 pk[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 16 * u;
                pk[u] = make_uint4(0, 0, 0, 0);
                if (live && c < nch) {
                    if (DT == 0) pk[u] = *reinterpret_cast<const uint4*>(static_cast<const float*>(store_) + off32(id, c, nkb));
                    else pk[u] = *reinterpret_cast<const uint4*>(static_cast<const uint16_t*>(store_) + off16(id, c, nkb));
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int c = c0 + 16 * u;
                if (c >= nch) break;
                const uint32_t w[4] = {pk[u].x, pk[u].y, pk[u].z, pk[u].w};
                if (DT == 0) {
                    const float4 y = *reinterpret_cast<const float4*>(q + c * 4);
                    const float yy[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) { double x = __uint_as_float(w[i]); dot += x * (double)yy[i]; ssq += x * x; }
                } else {
                    const float4 y0 = *reinterpret_cast<const float4*>(q + c * 8), y1 = *reinterpret_cast<const float4*>(q + c * 8 + 4);
                    const float yy[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint16_t lo = (uint16_t)(w[i] & 0xffff), hi = (uint16_t)(w[i] >> 16);
                        const double x0 = DT == 1 ? bf16_to_f(lo) : f16_to_f(lo);
                        const double x1 = DT == 1 ? bf16_to_f(hi) : f16_to_f(hi);
                        dot += x0 * (double)yy[2 * i] + x1 * (double)yy[2 * i + 1];
                        ssq += x0 * x0 + x1 * x1;
                    }
                }
            }
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) { dot += __shfl_xor(dot, o, 64); ssq += __shfl_xor(ssq, o, 64); }
        if (live && sub == 0) {
            const double sim = dot * invq64[b] * (1.0 / sqrt(ssq));
            if constexpr (REQUANT) surv[(int64_t)b * SURV_CAP + j] = pack_key(sim == sim ? (float)sim : -INFINITY, id);
            else exact[(int64_t)b * exact_stride + j] = sim;
        }
    }
}

// The selection after the last scan pass, with the refinement of a crowded band (see select_one_query).
constexpr float EXACT_KEY_MARGIN = 2.4e-7f;     // two fp32 roundings of a similarity of magnitude <= 1
template <int DT>
__device__ __forceinline__ void select_final_one_query(const int b, uint64_t* surv, uint32_t* cnt, float* thr,
                                                       const float* invq, uint32_t* counters, uint32_t* flags, int k1,
                                                       float margin, int may_have_empty, int keep_max,
                                                       const void* store_, const float* qf, const double* invq64, int nkb) {
    const bool crowded = select_one_query(b, surv, cnt, thr, invq, counters, flags, k1, margin, may_have_empty, keep_max, SEL_FINAL);
    __syncthreads();
    if (crowded) {                                  // uniform
        rescore_one_query<DT, true>(b, 0, 1, store_, qf, invq64, surv, cnt, nullptr, nkb, 0);
        __syncthreads();
        select_one_query(b, surv, cnt, thr, invq, counters, flags, k1, EXACT_KEY_MARGIN, may_have_empty, keep_max, SEL_EXACT);
        __syncthreads();
    }
}

template <int DT>
__global__ __launch_bounds__(1024) void k_select_final(uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt, float* __restrict__ thr,
                                                       const float* __restrict__ invq, uint32_t* __restrict__ counters,
                                                       uint32_t* __restrict__ flags, int k1, float margin, int may_have_empty,
                                                       int keep_max, const void* __restrict__ store_, const float* __restrict__ qf,
                                                       const double* __restrict__ invq64, int nkb) {
    select_final_one_query<DT>((int)blockIdx.x, surv, cnt, thr, invq, counters, flags, k1, margin, may_have_empty, keep_max,
                               store_, qf, invq64, nkb);
}

template <int DT>
__global__ __launch_bounds__(1024) void k_rescore(const void* __restrict__ store_, const float* __restrict__ qf,
                                                  const double* __restrict__ invq64, const uint64_t* __restrict__ surv,
                                                  const uint32_t* __restrict__ cnt, double* __restrict__ exact,
                                                  int nkb, int exact_stride) {
    rescore_one_query<DT>((int)blockIdx.x, (int)blockIdx.y, (int)gridDim.y, store_, qf, invq64, surv, cnt, exact, nkb, exact_stride);
}

// ---- exhaustive selection (mem_retrieve_exact): no threshold, no scan, no list that can overflow ----
// The bank is walked in ranges small enough that the carried candidates plus every row of the range fit
// a survivor list.  Per range: (1) the range's ids are appended to every query's list, (2) each appended
// entry gets its key from the similarity accumulated in fp64 (rounded to fp32), (3) the list is cut back to
// the k1 best keys plus those within two fp32 roundings of the k1-th (or, if that band is crowded, to
// exactly the k1 best: lower ids first among equal similarities).  The top-k1 of a union is the top-k1 of
// the parts' top-k1, so after the last range the list holds the pool.
__global__ __launch_bounds__(256) void k_exact_fill(uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt, int32_t first_id, int n_new) {
    const int b = (int)blockIdx.x;
    const uint32_t have = cnt[b];
    __syncthreads();                                    // every lane has read the old count
    for (int i = threadIdx.x; i < n_new; i += 256) surv[(int64_t)b * SURV_CAP + have + i] = pack_key(0.f, first_id + i);
    if (threadIdx.x == 0) cnt[b] = have + (uint32_t)n_new;
}

template <int DT>
__global__ __launch_bounds__(1024) void k_exact_keys(const void* __restrict__ store_, const float* __restrict__ qf,
                                                     const double* __restrict__ invq64, uint64_t* __restrict__ surv,
                                                     const uint32_t* __restrict__ cnt, int nkb, int n_new) {
    const int b = (int)blockIdx.x;
    rescore_one_query<DT, true>(b, (int)blockIdx.y, (int)gridDim.y, store_, qf, invq64, surv, cnt, nullptr, nkb, 0, (int)cnt[b] - n_new);
}

__global__ __launch_bounds__(1024) void k_exact_select(uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt, float* __restrict__ thr,
                                                       const float* __restrict__ invq, uint32_t* __restrict__ counters,
                                                       uint32_t* __restrict__ flags, int k1, int keep_max) {
    select_one_query((int)blockIdx.x, surv, cnt, thr, invq, counters, flags, k1, EXACT_KEY_MARGIN, 0, keep_max, SEL_EXACT);
}

constexpr int RERANK_T = 256;

// One block of the Philox-4x32 counter-based generator with 10 rounds (Salmon et al., SC'11): each
// round multiplies counter words 0 and 2 by fixed odd constants, crosses the high and low halves
// with the other two words and the key, and the key advances by fixed Weyl increments.
struct philox_out { uint32_t w0, w1, w2, w3; };
__device__ __forceinline__ philox_out philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                    uint32_t k0, uint32_t k1) {
    constexpr uint32_t MUL_A = 0xD2511F53u, MUL_B = 0xCD9E8D57u, WEYL_A = 0x9E3779B9u, WEYL_B = 0xBB67AE85u;
#pragma unroll
    for (int round = 0; round < 10; ++round) {
        const uint32_t a_hi = __umulhi(MUL_A, c0), a_lo = MUL_A * c0;
        const uint32_t b_hi = __umulhi(MUL_B, c2), b_lo = MUL_B * c2;
        c0 = b_hi ^ c1 ^ k0;
        c2 = a_hi ^ c3 ^ k1;
        c1 = b_lo;
        c3 = a_lo;
        k0 += WEYL_A;
        k1 += WEYL_B;
    }
    return {c0, c1, c2, c3};
}

// Parameters of the epsilon-greedy slot filling (Sec. 3.3); threshold 0 and no flag output = greedy.
struct EpsGreedy {
    uint64_t threshold;      // floor(eps * 2^32): a slot explores iff its first random word is below it
    uint64_t seed, step;
    unsigned char* explored; // [B][k2] or null
};

// Deterministic sum of one value per pool entry: wavefront butterflies, then the four partial sums of
// the first 256 lanes added in a fixed order.  `red` has four slots; pool entry i belongs to lane
// i < SMALL_K1_MAX = 256, so the lanes beyond (the fused kernel runs 1024) hold zeros and store nothing.
__device__ __forceinline__ double block_sum(double* red, int tid, double x) {
    static_assert(SMALL_K1_MAX == 4 * 64, "block_sum adds the partial sums of exactly four wavefronts");
    x = wave_sum_d(x);
    if ((tid & 63) == 0 && tid < SMALL_K1_MAX) red[tid >> 6] = x;
    __syncthreads();
    double r = (red[0] + red[1]) + (red[2] + red[3]);
    __syncthreads();
    return r;
}

// A NaN similarity or score (a zero-norm or non-finite row or query, a NaN in the Q table: inputs
// for which the results are unspecified) is ranked as -inf, so that the orderings below stay total
// orders: every rank is taken exactly once and every id that is gathered with is a real one.
__device__ __forceinline__ double finite_or_lowest(double v) { return v == v ? v : -INFINITY; }

// (v, id) before (w, jd)?  Written without short-circuit operators: inside the counting loops below
// the arguments come from LDS, and a short-circuit form compiles to a branch per element with the
// second LDS read behind it, so that every element pays two LDS round trips (measured: 200 cycles
// per element, 36 us for a 128-entry pool); this form lets the reads of an unrolled group go out together.
__device__ __forceinline__ bool ranks_before(double v, int32_t id, double w, int32_t jd) {
    return (bool)((int)(v > w) | ((int)(v == w) & (int)(id < jd)));
}

// Candidate pool and value filter for one query (Sec. 3.2): order the re-scored candidates by
// (similarity desc, id asc), keep k1 as the pool C(x); gather the stage's Q values; z-score both
// over the pool (population deviation, denominator std + 1e-6); score = (1-lambda) z_s + lambda z_q;
// emit the k2 best by (score desc, id asc).  All in fp64, scores rounded to fp32 on output.
// The lists are short (at most 512 and 256 entries), so both orderings are done by counting: every
// thread counts how many entries precede its own (each step reads one LDS entry, broadcast to all
// lanes) and writes its entry to that rank -- two barriers instead of a sorting network.
// T: lanes of the workgroup that runs it (256, or 1024 inside the fused kernel below; pool entry i belongs
// to lane i either way, and the block sums add the same four partial sums in the same order).
template <int T>
__device__ __forceinline__ void rerank_one_query(const int b, const uint64_t* surv, const uint32_t* cnt,
                                                const double* exact, const float* qstage,
                                                int k1, int k2, double lambda, int32_t* out_ids,
                                                float* out_scores, int32_t* cand_ids,
                                                float* cand_sims, EpsGreedy eg, int exact_stride) {
    __shared__ double v0[KEEP_MAX], v1[SMALL_K1_MAX];
    __shared__ int32_t i0[KEEP_MAX], i1[SMALL_K1_MAX];
    __shared__ double red[4];
    const int tid = threadIdx.x;
    const int kk = (int)cnt[b];
    for (int i = tid; i < kk; i += T) {
        v0[i] = finite_or_lowest(exact[(int64_t)b * exact_stride + i]);
        i0[i] = key_id(surv[(int64_t)b * SURV_CAP + i]);
    }
    __syncthreads();
    const int k1e = kk < k1 ? kk : k1;
    // ordering 1: the k1e best by (similarity desc, id asc) -> (v1, i1)
    // (SPLIT lanes share an entry when the workgroup has lanes to spare: each counts over every
    // SPLIT-th other entry and the partial counts are added across the neighbouring lanes)
    constexpr int SPLIT = T >= 1024 ? 4 : 1;
    for (int i = tid / SPLIT; i < kk; i += T / SPLIT) {           // trip count uniform within a lane group
        const double v = v0[i];
        const int32_t id = i0[i];
        int rank = 0;
#pragma unroll 8
        for (int j = tid % SPLIT; j < kk; j += SPLIT) rank += ranks_before(v0[j], i0[j], v, id);
        if (SPLIT == 4) { rank += __shfl_xor(rank, 1, 64); rank += __shfl_xor(rank, 2, 64); }
        if (tid % SPLIT == 0 && rank < k1e) { v1[rank] = v; i1[rank] = id; }
    }
    __syncthreads();
    if (cand_ids)
        for (int i = tid; i < k1; i += T) {
            cand_ids[(int64_t)b * k1 + i] = i < k1e ? i1[i] : -1;
            cand_sims[(int64_t)b * k1 + i] = i < k1e ? (float)v1[i] : -INFINITY;
        }
    // z-scores over the pool (one pool entry per thread, k1e <= 256)
    const bool mine = tid < k1e;
    const double sim = mine ? v1[tid] : 0.0;
    const int32_t id = mine ? i1[tid] : 0x7fffffff;
    const double qv = mine ? (double)qstage[id] : 0.0;
    double score = -INFINITY;
    if (k1e > 0) {                                                    // uniform
        const double mean_s = block_sum(red, tid, sim) / k1e;
        const double mean_q = block_sum(red, tid, qv) / k1e;
        const double ds = mine ? sim - mean_s : 0.0, dq = mine ? qv - mean_q : 0.0;
        const double var_s = block_sum(red, tid, ds * ds) / k1e;
        const double var_q = block_sum(red, tid, dq * dq) / k1e;
        const double scale_s = 1.0 / (sqrt(var_s) + 1e-6), scale_q = 1.0 / (sqrt(var_q) + 1e-6);
        if (mine) score = finite_or_lowest((1.0 - lambda) * (ds * scale_s) + lambda * (dq * scale_q));
    }
    __syncthreads();
    // ordering 2: the k2 best by (score desc, id asc); v0/i0 are reused for the scores
    if (mine) { v0[tid] = score; i0[tid] = id; }
    __syncthreads();
    const int k2e = k1e < k2 ? k1e : k2;
    const bool greedy = eg.threshold == 0 && eg.explored == nullptr;
    int rank = 0;
    if (mine) {
#pragma unroll 8
        for (int j = 0; j < k1e; ++j) rank += ranks_before(v0[j], i0[j], score, id);
        if (greedy && rank < k2e) { out_ids[(int64_t)b * k2 + rank] = id; out_scores[(int64_t)b * k2 + rank] = (float)score; }
    }
    for (int i = k2e + tid; i < k2; i += T) {
        out_ids[(int64_t)b * k2 + i] = -1;
        out_scores[(int64_t)b * k2 + i] = -INFINITY;
        if (eg.explored) eg.explored[(int64_t)b * k2 + i] = 0;
    }
    if (greedy) return;                                               // uniform

    // Epsilon-greedy slot filling (Sec. 3.3).  The whole pool is laid out in greedy order; every
    // slot's draw is computed by its own lane (the draws depend on the slot number only); then one
    // lane fills the slots in order, because which members are still free depends on the slots before.
    __shared__ uint32_t word0[SMALL_K1_MAX], word1[SMALL_K1_MAX];
    if (mine) { v1[rank] = score; i1[rank] = id; }
    if (tid < k2e) {
        const philox_out r = philox4x32_10((uint32_t)eg.step, (uint32_t)(eg.step >> 32), (uint32_t)b, (uint32_t)tid,
                                           (uint32_t)eg.seed, (uint32_t)(eg.seed >> 32));
        word0[tid] = r.w0;
        word1[tid] = r.w1;
    }
    __syncthreads();
    if (tid == 0) {
        uint64_t taken[SMALL_K1_MAX / 64];                     // bit set = chosen (or past the pool's end)
#pragma unroll
        for (int w = 0; w < SMALL_K1_MAX / 64; ++w) {
            const int lo = w * 64;
            taken[w] = k1e >= lo + 64 ? 0ull : k1e <= lo ? ~0ull : (~0ull << (k1e - lo));
        }
        for (int j = 0; j < k2e; ++j) {
            const bool explore = (uint64_t)word0[j] < eg.threshold;
            const uint32_t remaining = (uint32_t)(k1e - j);
            int want = explore ? (int)(((uint64_t)word1[j] * remaining) >> 32) : 0;   // index among the free members
            int pos = 0;
#pragma unroll
            for (int w = 0; w < SMALL_K1_MAX / 64; ++w) {
                uint64_t fr = ~taken[w];
                const int c = __popcll(fr);
                if (want >= 0 && want < c) {
                    for (int t = 0; t < want; ++t) fr &= fr - 1;              // drop the `want` lowest free bits
                    const int bit = __ffsll((long long)fr) - 1;
                    taken[w] |= 1ull << bit;
                    pos = w * 64 + bit;
                    want = -1;
                } else if (want >= 0) {
                    want -= c;
                }
            }
            out_ids[(int64_t)b * k2 + j] = i1[pos];
            out_scores[(int64_t)b * k2 + j] = (float)v1[pos];
            if (eg.explored) eg.explored[(int64_t)b * k2 + j] = explore ? 1 : 0;
        }
    }
}


__global__ __launch_bounds__(RERANK_T) void k_rerank(const uint64_t* __restrict__ surv, const uint32_t* __restrict__ cnt,
                                                const double* __restrict__ exact, const float* __restrict__ qstage,
                                                int k1, int k2, double lambda, int32_t* __restrict__ out_ids,
                                                float* __restrict__ out_scores, int32_t* __restrict__ cand_ids,
                                                float* __restrict__ cand_sims, EpsGreedy eg, int exact_stride) {
    rerank_one_query<RERANK_T>((int)blockIdx.x, surv, cnt, exact, qstage, k1, k2, lambda, out_ids, out_scores, cand_ids, cand_sims, eg, exact_stride);
}

// The last selection, the exact re-scoring and the value filter of one query in one launch (pools of up
// to 128, one workgroup per query): the three steps hand their results on through the same global
// buffers as the separate kernels do -- a workgroup's own writes are visible to it after a barrier --
// so the results are bit for bit those of the three launches, without two launch latencies.
template <int DT>
__global__ __launch_bounds__(1024) void k_select_rescore_rerank(
        uint64_t* __restrict__ surv, uint32_t* __restrict__ cnt, float* __restrict__ thr, const float* __restrict__ invq,
        uint32_t* __restrict__ counters, uint32_t* __restrict__ flags, int k1, float margin, int may_have_empty, int keep_max,
        const void* __restrict__ store_, const float* __restrict__ qf, const double* __restrict__ invq64,
        double* __restrict__ exact, int nkb, int exact_stride,
        const float* __restrict__ qstage, int k2, double lambda, int32_t* __restrict__ out_ids, float* __restrict__ out_scores,
        int32_t* __restrict__ cand_ids, float* __restrict__ cand_sims, EpsGreedy eg) {
    const int b = (int)blockIdx.x;
    select_final_one_query<DT>(b, surv, cnt, thr, invq, counters, flags, k1, margin, may_have_empty, keep_max, store_, qf, invq64, nkb);
    rescore_one_query<DT>(b, 0, 1, store_, qf, invq64, surv, cnt, exact, nkb, exact_stride);
    __syncthreads();
    rerank_one_query<1024>(b, surv, cnt, exact, qstage, k1, k2, lambda, out_ids, out_scores, cand_ids, cand_sims, eg, exact_stride);
}

}  // namespace evk
