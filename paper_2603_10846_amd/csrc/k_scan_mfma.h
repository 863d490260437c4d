// Similarity scan for query batches large enough to be a dense contraction (Sec. 3.2, dense
// recall): scores[q][n] = <query q, bank row n> on the matrix cores, never written to memory.
//
// A workgroup of 4 wavefronts owns one 256-row bank tile and QT queries.  Per k-block the bank
// tile's 32 KB block (already in LDS operand order in HBM, see layout.h) and the queries' block are
// staged in LDS, double buffered, and consumed by v_mfma_f32_32x32x16 (bf16 or f16 operands, fp32
// accumulation).  Queries are the rows of the accumulator tile and bank rows its columns, so a lane
// holds one bank row per 32x32 block and the per-row inverse norm is a per-lane constant.
//
// fp32 stores: each value is split on the fly into bf16 hi + bf16 lo and the product is
// hi*hi + hi*lo + lo*hi (three MFMAs, relative error of a product about 2^-16); this only has to
// be good enough for the filter, since the value filter re-scores the selected candidates in fp64.
//
// Epilogue: score * invnorm[row] is compared with the query's threshold (pre-divided by the
// query's inverse norm); the rare survivors are appended to the query's list.
#pragma once
#include "k_scan_gemv.h"
#include "layout.h"

namespace evk {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;

template <int DT>
__device__ __forceinline__ f32x16_t mfma32(u32x4_t a, u32x4_t b, f32x16_t c) {
    if constexpr (DT == 2) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8_t, a), __builtin_bit_cast(f16x8_t, b), c, 0, 0, 0);
    } else {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
    }
}

__device__ __forceinline__ uint32_t pack_bf16x2_hi(float a, float b, float& ra, float& rb) {
    uint16_t ha = f2bf16_rne(a), hb = f2bf16_rne(b);
    ra = a - bf16_to_f(ha); rb = b - bf16_to_f(hb);
    return ha | ((uint32_t)hb << 16);
}

constexpr int STAGE_BANK_BYTES = TILE_ROWS * 128;

// LDS: two stages (bank tile + query tile), then per-query threshold, inverse norm, survivor count
// and list base, then one counter.  After the k-loop the stage area is reused as the workgroup's
// survivor list (8-byte key + 4-byte query index per entry).
template <int QT> constexpr int scan_mfma_lds_bytes() { return 2 * (STAGE_BANK_BYTES + QT * 128) + QT * 16 + 16; }
template <int QT> constexpr int scan_mfma_list_cap() {
    int c = 2 * (STAGE_BANK_BYTES + QT * 128) / 12 / 256 * 256;
    return c > 8192 ? 8192 : c;
}

// DT: 0 fp32 store (bf16 split), 1 bf16, 2 f16.  Wave grid WQ x WR, each wave MQ x MR blocks of 32x32.
template <int DT, int MQ, int WQ, int MR, int WR>
__global__ __launch_bounds__(256) void k_scan_mfma(const void* __restrict__ store_, const float* __restrict__ invnorm,
                                                   const uint16_t* __restrict__ qop, const float* __restrict__ invq,
                                                   const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                   uint64_t* __restrict__ surv, int64_t N, int nkb, int Bp,
                                                   Level L) {
    static_assert(WQ * WR == 4 && MR * WR == 8, "4 waves, 256 bank rows per workgroup");
    constexpr int QT = 32 * MQ * WQ;
    constexpr int QCH = QT / 32;                       // 16-byte query chunks per lane per stage
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wq = wave / WR, wr = wave % WR;

    // blockIdx -> (bank tile, query tile): workgroups that share a bank tile get consecutive slots
    // of one XCD (blocks are dealt to the 8 XCDs round-robin), so the tile is fetched from HBM once
    // and the other query tiles hit that XCD's L2.
    const int nqt = Bp / QT;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int qt = slot % nqt;
    const int j = (slot / nqt) * 8 + xcd;
    if (j >= L.ntiles) return;
    const int64_t t = level_tile(L, j);
    const int q0 = qt * QT;

    constexpr int STAGE_BYTES = STAGE_BANK_BYTES + QT * 128;
    auto sbank = [&](int s) { return smem + s * STAGE_BYTES; };
    auto sq = [&](int s) { return smem + s * STAGE_BYTES + STAGE_BANK_BYTES; };
    float* thr_s = reinterpret_cast<float*>(smem + 2 * STAGE_BYTES);
    float* invq_s = thr_s + QT;
    uint32_t* cnt_s = reinterpret_cast<uint32_t*>(invq_s + QT);
    uint32_t* base_s = cnt_s + QT;
    uint32_t* total_s = base_s + QT;
    for (int i = tid; i < QT; i += 256) { thr_s[i] = thr[q0 + i]; invq_s[i] = invq[q0 + i]; cnt_s[i] = 0; }
    if (tid == 0) *total_s = 0;

    f32x16_t acc[MQ][MR];
#pragma unroll
    for (int a = 0; a < MQ; ++a)
#pragma unroll
        for (int b = 0; b < MR; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int nsteps = DT == 0 ? nkb * 2 : nkb;
    u32x4_t gb[8], gq[QCH];

    auto gload = [&](int step) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
            const float* blk = static_cast<const float*>(store_) + (t * nkb + (step >> 1)) * (int64_t)BLOCK_ELEMS + (step & 1) * 32;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int g = i * 256 + tid, r = g >> 3, c4 = g & 7;
                gb[i] = *reinterpret_cast<const u32x4_t*>(blk + r * KB + c4 * 4);
            }
        } else {
            const uint16_t* blk = static_cast<const uint16_t*>(store_) + (t * nkb + step) * (int64_t)BLOCK_ELEMS;
#pragma unroll
            for (int i = 0; i < 8; ++i) gb[i] = *reinterpret_cast<const u32x4_t*>(blk + (i * 256 + tid) * 8);
        }
        const uint16_t* qb = qop + ((int64_t)step * Bp + q0) * KB;
#pragma unroll
        for (int i = 0; i < QCH; ++i) gq[i] = *reinterpret_cast<const u32x4_t*>(qb + (i * 256 + tid) * 8);
    };
    auto lstore = [&](int s) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                int g = i * 256 + tid, r = g >> 3, c4 = g & 7;
                float f0 = __uint_as_float(gb[i].x), f1 = __uint_as_float(gb[i].y);
                float f2 = __uint_as_float(gb[i].z), f3 = __uint_as_float(gb[i].w);
                float r0, r1, r2, r3;
                u32x2_t hi, lo;
                hi.x = pack_bf16x2_hi(f0, f1, r0, r1); hi.y = pack_bf16x2_hi(f2, f3, r2, r3);
                lo.x = f2bf16_rne(r0) | ((uint32_t)f2bf16_rne(r1) << 16);
                lo.y = f2bf16_rne(r2) | ((uint32_t)f2bf16_rne(r3) << 16);
                unsigned char* rowp = sbank(s) + r * 128 + (c4 & 1) * 8;
                *reinterpret_cast<u32x2_t*>(rowp + swz16(c4 >> 1, r) * 16) = hi;
                *reinterpret_cast<u32x2_t*>(rowp + swz16(4 + (c4 >> 1), r) * 16) = lo;
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) *reinterpret_cast<u32x4_t*>(sbank(s) + (i * 256 + tid) * 16) = gb[i];
        }
#pragma unroll
        for (int i = 0; i < QCH; ++i) *reinterpret_cast<u32x4_t*>(sq(s) + (i * 256 + tid) * 16) = gq[i];
    };
    auto frag = [&](const unsigned char* base, int row, int chunk) __attribute__((always_inline)) {
        return *reinterpret_cast<const u32x4_t*>(base + row * 128 + swz16(chunk, row) * 16);
    };
    auto compute = [&](int s) __attribute__((always_inline)) {
        const int half = lane >> 5, l32 = lane & 31;
        if constexpr (DT == 0) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4_t ah[MQ], al[MQ], bh[MR], bl[MR];
#pragma unroll
                for (int a = 0; a < MQ; ++a) {
                    int row = (wq * MQ + a) * 32 + l32;
                    ah[a] = frag(sq(s), row, 2 * ks + half); al[a] = frag(sq(s), row, 4 + 2 * ks + half);
                }
#pragma unroll
                for (int b = 0; b < MR; ++b) {
                    int row = (wr * MR + b) * 32 + l32;
                    bh[b] = frag(sbank(s), row, 2 * ks + half); bl[b] = frag(sbank(s), row, 4 + 2 * ks + half);
                }
#pragma unroll
                for (int a = 0; a < MQ; ++a)
#pragma unroll
                    for (int b = 0; b < MR; ++b) {
                        acc[a][b] = mfma32<1>(al[a], bh[b], acc[a][b]);
                        acc[a][b] = mfma32<1>(ah[a], bl[b], acc[a][b]);
                        acc[a][b] = mfma32<1>(ah[a], bh[b], acc[a][b]);
                    }
            }
        } else {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                u32x4_t af[MQ], bf[MR];
#pragma unroll
                for (int a = 0; a < MQ; ++a) af[a] = frag(sq(s), (wq * MQ + a) * 32 + l32, 2 * ks + half);
#pragma unroll
                for (int b = 0; b < MR; ++b) bf[b] = frag(sbank(s), (wr * MR + b) * 32 + l32, 2 * ks + half);
#pragma unroll
                for (int a = 0; a < MQ; ++a)
#pragma unroll
                    for (int b = 0; b < MR; ++b) acc[a][b] = mfma32<DT>(af[a], bf[b], acc[a][b]);
            }
        }
    };

    gload(0);
    lstore(0);
    __syncthreads();
    for (int step = 0; step < nsteps; ++step) {
        const int s = step & 1;
        if (step + 1 < nsteps) gload(step + 1);
        compute(s);
        if (step + 1 < nsteps) lstore(s ^ 1);
        __syncthreads();
    }

    // ---- epilogue ----
    const int half = lane >> 5, l32 = lane & 31;
    if (L.rho == 0) {
        // Sparsest pass: no threshold yet, every row is kept.  Slot = position of the row in this
        // pass, so no counter is needed (the count was preset to the pass's number of valid rows).
#pragma unroll
        for (int b = 0; b < MR; ++b) {
            const int rt = (wr * MR + b) * 32 + l32;
            const int64_t id = t * TILE_ROWS + rt;
            if (id >= N) continue;
            const float inve = invnorm[id];
            const int64_t pos = (int64_t)j * TILE_ROWS + rt;
#pragma unroll
            for (int a = 0; a < MQ; ++a)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int ql = (wq * MQ + a) * 32 + 4 * half + 8 * (r >> 2) + (r & 3);
                    surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = pack_key(acc[a][b][r] * inve * invq_s[ql], (int32_t)id);
                }
        }
        return;
    }
    // Filter against the per-query thresholds.  Survivors (rare) go to a workgroup list in LDS first,
    // so that the global slot counters are bumped once per (workgroup, query) and all at the same
    // time, instead of one dependent device-wide atomic per survivor.
    constexpr int LCAP = scan_mfma_list_cap<QT>();
    uint64_t* lkey = reinterpret_cast<uint64_t*>(smem);
    uint32_t* lq = reinterpret_cast<uint32_t*>(smem + LCAP * 8);
#pragma unroll
    for (int b = 0; b < MR; ++b) {
        const int64_t id = t * TILE_ROWS + (wr * MR + b) * 32 + l32;
        const bool valid = id < N;
        const float inve = valid ? invnorm[id] : 0.f;
#pragma unroll
        for (int a = 0; a < MQ; ++a) {
            const int qb = (wq * MQ + a) * 32 + 4 * half;     // local query of register 0
            uint32_t m = 0;
            float v[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                v[r] = acc[a][b][r] * inve;
                m |= (uint32_t)(v[r] >= thr_s[qb + 8 * (r >> 2) + (r & 3)]) << r;
            }
            if (!valid) m = 0;
            if (m) {
                uint32_t slot = atomicAdd(total_s, (uint32_t)__popc(m));
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (m & (1u << r)) {
                        const int ql = qb + 8 * (r >> 2) + (r & 3);
                        const uint64_t key = pack_key(v[r] * invq_s[ql], (int32_t)id);
                        if (slot < (uint32_t)LCAP) { lkey[slot] = key; lq[slot] = (uint32_t)ql; }
                        else {   // list full (a very loose threshold): fall back to the direct path
                            uint32_t pos = atomicAdd(cnt + q0 + ql, 1u);
                            if (pos < (uint32_t)SURV_CAP) surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = key;
                        }
                        ++slot;
                    }
            }
        }
    }
    __syncthreads();
    const uint32_t total = *total_s < (uint32_t)LCAP ? *total_s : (uint32_t)LCAP;
    for (uint32_t e = tid; e < total; e += 256) {
        uint32_t ql = lq[e];
        lq[e] = ql | (atomicAdd(cnt_s + ql, 1u) << 16);        // rank within this workgroup's entries of ql
    }
    __syncthreads();
    for (int i = tid; i < QT; i += 256) { uint32_t c = cnt_s[i]; base_s[i] = c ? atomicAdd(cnt + q0 + i, c) : 0u; }
    __syncthreads();
    for (uint32_t e = tid; e < total; e += 256) {
        uint32_t ql = lq[e] & 0xffffu, rank = lq[e] >> 16;
        uint32_t pos = base_s[ql] + rank;
        if (pos < (uint32_t)SURV_CAP) surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = lkey[e];
    }
}

}  // namespace evk
