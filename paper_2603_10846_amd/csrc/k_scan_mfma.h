// Similarity scan for query batches large enough to be a dense contraction (Sec. 3.2, dense
// recall): scores[q][n] = <query q, bank row n> on the matrix cores, never written to memory.
//
// Persistent workgroups of 4 wavefronts; each owns QT queries and walks over 256-row bank tiles.
// Per k-block the bank tile's 32 KB block (already in LDS operand order in HBM, see layout.h) and
// the queries' block are staged in LDS (two stages) and consumed by v_mfma_f32_32x32x16 (bf16 or
// f16 operands, fp32 accumulation).  Global loads run two k-blocks ahead of the MFMAs through two
// register sets, and the (tile, k-block) sequence is flattened, so the loads of the next tile are
// already in flight while a tile's epilogue runs.  Queries are the rows of the accumulator tile and
// bank rows its columns: a lane holds one bank row per 32x32 block and the row's inverse norm is a
// per-lane constant in the epilogue.
//
// fp32 stores: each value is split on the fly into bf16 hi + bf16 lo and the product is
// hi*hi + hi*lo + lo*hi (three MFMAs, relative error of a product about 2^-16); this only has to
// be good enough for the filter, since the value filter re-scores the selected candidates in fp64.
//
// Epilogue: score * invnorm[row] is compared with the query's threshold (pre-divided by the
// query's inverse norm); the rare survivors are appended to the query's list.
#pragma once
#include <type_traits>

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

// Bitwise OR of a value over the 64 lanes of a wavefront, returned as a wavefront-uniform value:
// shifts within rows of 16 lanes, then the row broadcasts, then lane 63 is read.
__device__ __forceinline__ uint32_t wave_or(uint32_t x) {
    int v = (int)x;
    v |= __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v |= __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v |= __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v |= __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8  -> lane 15 of each row
    v |= __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true);   // row_bcast:15 into rows 1 and 3
    v |= __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true);   // row_bcast:31 into rows 2 and 3
    return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}

constexpr int STAGE_BANK_BYTES = TILE_ROWS * 128;
constexpr int SCAN_LIST_CAP = 2048;     // survivor entries a workgroup can stage per tile

// LDS: two stages (bank tile + query tile); per-query threshold, inverse norm, survivor count and
// list base; the workgroup's survivor list (8-byte key + 4-byte query index per entry); a counter.
template <int QT> constexpr int scan_mfma_lds_bytes() {
    return 2 * (STAGE_BANK_BYTES + QT * 128) + QT * 16 + SCAN_LIST_CAP * 12 + 16;
}

// DT: 0 fp32 store (bf16 split), 1 bf16, 2 f16.  Wave grid WQ x WR, each wave MQ x MR blocks of 32x32.
// gridDim.x is a multiple of 8 * (Bp / QT).
template <int DT, int MQ, int WQ, int MR, int WR>
__global__ __launch_bounds__(64 * WQ * WR) void k_scan_mfma(const void* __restrict__ store_, const float* __restrict__ invnorm,
                                                   const uint16_t* __restrict__ qop, const float* __restrict__ invq,
                                                   const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                   uint64_t* __restrict__ surv, int64_t N, int nkb, int Bp,
                                                   Level L, int flush_every) {
    static_assert((WQ * WR == 4 || WQ * WR == 8) && MR * WR == 8, "4 or 8 waves, 256 bank rows per workgroup");
    constexpr int NT = 64 * WQ * WR;                   // lanes per workgroup
    constexpr int QT = 32 * MQ * WQ;
    constexpr int BCH = 2048 / NT;                     // 16-byte bank chunks per lane per stage
    constexpr int QCH = QT * 8 / NT;                   // 16-byte query chunks per lane per stage
    constexpr int STAGE_BYTES = STAGE_BANK_BYTES + QT * 128;
    // 16-bit float type of the MFMA operands (bf16 also for fp32 stores, which are split into bf16)
    auto enc16 = [](float x) __attribute__((always_inline)) { return DT == 2 ? f2f16_rne(x) : f2bf16_rne(x); };
    auto dec16 = [](uint16_t h) __attribute__((always_inline)) { return DT == 2 ? f16_to_f(h) : bf16_to_f(h); };
    extern __shared__ __align__(16) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wq = wave / WR, wr = wave % WR;
    const int half = lane >> 5, l32 = lane & 31;

    // Workgroup -> (query tile, sequence of bank tiles).  Blocks are dealt to the 8 XCDs round-robin;
    // the nqt workgroups that share a bank tile are neighbours on one XCD and walk the tiles in the
    // same order, so a tile is fetched from HBM once and the other query tiles hit that XCD's L2.
    const int nqt = Bp / QT;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int qt = slot % nqt, group = slot / nqt;
    const int groups = (gridDim.x >> 3) / nqt;         // tile walkers per XCD
    const int q0 = qt * QT;
    // tiles of this workgroup: j = (group + i * groups) * 8 + xcd < L.ntiles
    const int first_j = group * 8 + xcd, stride_j = groups * 8;
    if (first_j >= L.ntiles) return;
    const int my_tiles = (L.ntiles - first_j + stride_j - 1) / stride_j;

    auto sbank = [&](int s) __attribute__((always_inline)) { return smem + s * STAGE_BYTES; };
    auto sq = [&](int s) __attribute__((always_inline)) { return smem + s * STAGE_BYTES + STAGE_BANK_BYTES; };
    uint32_t* thp_s = reinterpret_cast<uint32_t*>(smem + 2 * STAGE_BYTES);   // thresholds as (hi | lo << 16), 16-bit floats
    float* invq_s = reinterpret_cast<float*>(thp_s + QT);
    uint32_t* cnt_s = reinterpret_cast<uint32_t*>(invq_s + QT);
    uint32_t* base_s = cnt_s + QT;
    uint64_t* lkey = reinterpret_cast<uint64_t*>(base_s + QT);
    uint32_t* lq = reinterpret_cast<uint32_t*>(lkey + SCAN_LIST_CAP);
    uint32_t* total_s = lq + SCAN_LIST_CAP;
    for (int i = tid; i < QT; i += NT) {
        const float th = thr[q0 + i];
        const uint16_t hi = enc16(th), lo = enc16(th - dec16(hi));
        thp_s[i] = hi | ((uint32_t)lo << 16);
        invq_s[i] = invq[q0 + i];
        cnt_s[i] = 0;
    }
    if (tid == 0) *total_s = 0;

    // Accumulators: (re)initialised at the start of every tile by MFMAs with a zero C operand.
    // (An explicit re-zeroing inside the tile loop makes the compiler keep two copies of them.)
    f32x16_t acc[MQ][MR];

    // Steps per tile, made even so that the two register sets / LDS stages are in the same phase at
    // every tile boundary: an odd count gets one dummy step that multiplies the tile's last bank
    // block with an all-zero query block (the query operand holds one such block at index nkb).
    const int real_steps = DT == 0 ? nkb * 2 : nkb;
    const int nsteps = real_steps + (real_steps & 1);
    u32x4_t gbA[BCH], gbB[BCH], gqA[QCH], gqB[QCH];

    // Bank and query loads run two steps ahead of the MFMAs.
    // Each workgroup starts its k-loop at a different k-block (the order of the k-blocks does not
    // matter for a dot product): workgroups run in near lock-step over tiles that are 2^n bytes
    // apart, and without the rotation they would all pull from the same few HBM channels at once.
    const int rot = (int)((blockIdx.x * 7u) % (unsigned)real_steps);
    auto rotated = [&](int step) __attribute__((always_inline)) {   // logical step -> k-step actually loaded
        if (step >= real_steps) return step;                          // the dummy step stays last
        int k = step + rot;
        return k >= real_steps ? k - real_steps : k;
    };
    int ld_ti = 0, ld_step = 0, ldq_step = 0;
    auto gload_q = [&](u32x4_t (&gq)[QCH]) __attribute__((always_inline)) {
        const uint16_t* qb = qop + ((int64_t)rotated(ldq_step) * Bp + q0) * KB;
#pragma unroll
        for (int i = 0; i < QCH; ++i) gq[i] = *reinterpret_cast<const u32x4_t*>(qb + (i * NT + tid) * 8);
        if (++ldq_step == nsteps) ldq_step = 0;
    };
    // first element of the bank tile the load cursor is on (recomputed only when the cursor moves on
    // to another tile: level_tile() contains an integer division)
    int64_t ld_tile_elem = level_tile(L, first_j) * nkb * (int64_t)BLOCK_ELEMS;
    auto gload = [&](u32x4_t (&gb)[BCH]) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
            const float* blk = static_cast<const float*>(store_) + ld_tile_elem + (rotated(ld_step) >> 1) * (int64_t)BLOCK_ELEMS + (rotated(ld_step) & 1) * 32;
#pragma unroll
            for (int i = 0; i < BCH; ++i) {
                int g = i * NT + tid, r = g >> 3, c4 = g & 7;
                gb[i] = *reinterpret_cast<const u32x4_t*>(blk + r * KB + c4 * 4);
            }
        } else {
            const int kb = ld_step < real_steps ? rotated(ld_step) : real_steps - 1;
            const uint16_t* blk = static_cast<const uint16_t*>(store_) + ld_tile_elem + kb * (int64_t)BLOCK_ELEMS;
#pragma unroll
            for (int i = 0; i < BCH; ++i) gb[i] = *reinterpret_cast<const u32x4_t*>(blk + (i * NT + tid) * 8);
        }
        // past the last step the cursor stays on the last tile: the two loads issued there are never
        // consumed, but keeping every phase free of branches lets the loads stay in flight across it
        if (++ld_step == nsteps) {
            ld_step = 0;
            if (ld_ti + 1 < my_tiles) { ++ld_ti; ld_tile_elem = level_tile(L, first_j + ld_ti * stride_j) * nkb * (int64_t)BLOCK_ELEMS; }
        }
    };
    auto lstore = [&](int s, u32x4_t (&gb)[BCH], u32x4_t (&gq)[QCH]) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
#pragma unroll
            for (int i = 0; i < BCH; ++i) {
                int g = i * NT + tid, r = g >> 3, c4 = g & 7;
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
            for (int i = 0; i < BCH; ++i) *reinterpret_cast<u32x4_t*>(sbank(s) + (i * NT + tid) * 16) = gb[i];
        }
#pragma unroll
        for (int i = 0; i < QCH; ++i) *reinterpret_cast<u32x4_t*>(sq(s) + (i * NT + tid) * 16) = gq[i];
    };
    // Operand addresses.  Row (block*32 + l32) of an operand tile, logical chunk c = 2*k4 + half:
    // byte offset = block*4096 + l32*128 + ((c ^ f(l32)) * 16), the swizzle depending on l32 only.
    // So four per-lane offsets per operand (k4 = 0..3, the wave's first block folded in) serve every
    // block, both stages and all k-steps; the rest of the address is a compile-time constant.
    uint32_t offA[4], offB[4];
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) {
        const uint32_t o = l32 * 128 + swz16(2 * k4 + half, l32) * 16;
        offA[k4] = o + STAGE_BANK_BYTES + wq * MQ * 4096;
        offB[k4] = o + wr * MR * 4096;
    }
    auto frag = [&](int s, uint32_t off, int block) __attribute__((always_inline)) {
        return *reinterpret_cast<const u32x4_t*>(smem + off + (s * STAGE_BYTES + block * 4096));
    };
    // `mid` (the LDS stores of the next step's operands) runs between the second and third k-step, so
    // that those stores overlap the MFMAs instead of forming a separate period before the barrier.
    auto compute = [&](int s, auto mid) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                u32x4_t ah[MQ], al[MQ], bh[MR], bl[MR];
#pragma unroll
                for (int a = 0; a < MQ; ++a) { ah[a] = frag(s, offA[ks], a); al[a] = frag(s, offA[2 + ks], a); }
#pragma unroll
                for (int b = 0; b < MR; ++b) { bh[b] = frag(s, offB[ks], b); bl[b] = frag(s, offB[2 + ks], b); }
#pragma unroll
                for (int a = 0; a < MQ; ++a)
#pragma unroll
                    for (int b = 0; b < MR; ++b) {
                        acc[a][b] = mfma32<1>(al[a], bh[b], acc[a][b]);
                        acc[a][b] = mfma32<1>(ah[a], bl[b], acc[a][b]);
                        acc[a][b] = mfma32<1>(ah[a], bh[b], acc[a][b]);
                    }
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 0) { mid(); __builtin_amdgcn_sched_barrier(0); }
            }
        } else {
            // Operand fragments are double buffered by hand (those of k-step ks+1 are read from LDS
            // while the MFMAs of ks run) and the scheduler is fenced per k-step, which bounds the
            // live fragment registers to two k-steps' worth.
            // (With two wavefronts per SIMD the other wavefront's MFMAs cover the LDS latency, and the
            // registers are better spent on loads in flight: fragments are then single buffered.)
            constexpr int FB = NT == 512 ? 0 : 1;      // index mask of the fragment buffers
            u32x4_t af[FB + 1][MQ], bf[FB + 1][MR];
#pragma unroll
            for (int a = 0; a < MQ; ++a) af[0][a] = frag(s, offA[0], a);
#pragma unroll
            for (int b = 0; b < MR; ++b) bf[0][b] = frag(s, offB[0], b);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks < 3 && FB) {
#pragma unroll
                    for (int a = 0; a < MQ; ++a) af[(ks + 1) & FB][a] = frag(s, offA[ks + 1], a);
#pragma unroll
                    for (int b = 0; b < MR; ++b) bf[(ks + 1) & FB][b] = frag(s, offB[ks + 1], b);
                }
#pragma unroll
                for (int a = 0; a < MQ; ++a)
#pragma unroll
                    for (int b = 0; b < MR; ++b) {
                        acc[a][b] = mfma32<DT>(af[ks & FB][a], bf[ks & FB][b], acc[a][b]);
                    }
                __builtin_amdgcn_sched_barrier(0);
                if (ks == 1) { mid(); __builtin_amdgcn_sched_barrier(0); }
                if (ks < 3 && !FB) {
#pragma unroll
                    for (int a = 0; a < MQ; ++a) af[0][a] = frag(s, offA[ks + 1], a);
#pragma unroll
                    for (int b = 0; b < MR; ++b) bf[0][b] = frag(s, offB[ks + 1], b);
                }
            }
        }
    };

    // Write the workgroup's staged survivors to the per-query lists (all lanes call it together):
    // rank the entries of each query with LDS atomics, reserve that many slots with one device-wide
    // integer atomic per query that has any, copy.
    auto flush = [&]() __attribute__((always_inline)) {
        const uint32_t total = *total_s < (uint32_t)SCAN_LIST_CAP ? *total_s : (uint32_t)SCAN_LIST_CAP;
        for (uint32_t e = tid; e < total; e += NT) {
            uint32_t ql = lq[e];
            lq[e] = ql | (atomicAdd(cnt_s + ql, 1u) << 16);   // rank among the staged entries of ql
        }
        __syncthreads();
        for (int i = tid; i < QT; i += NT) {
            uint32_t c = cnt_s[i];
            base_s[i] = c ? atomicAdd(cnt + q0 + i, c) : 0u;
            cnt_s[i] = 0;
        }
        __syncthreads();
        for (uint32_t e = tid; e < total; e += NT) {
            uint32_t ql = lq[e] & 0xffffu, rank = lq[e] >> 16;
            uint32_t pos = base_s[ql] + rank;
            if (pos < (uint32_t)SURV_CAP) surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = lkey[e];
        }
        __syncthreads();
        if (tid == 0) *total_s = 0;
        __syncthreads();
    };

    // Inverse norms of this lane's MR bank rows: inv_r for the current tile, inv_n for the next one
    // (loaded a whole tile ahead, so they have long arrived when a tile starts).
    float inv_r[MR], inv_n[MR];
    auto load_invnorm = [&](int ti) __attribute__((always_inline)) {
        const int64_t t = level_tile(L, first_j + (ti < my_tiles ? ti : my_tiles - 1) * stride_j);
#pragma unroll
        for (int b = 0; b < MR; ++b) {
            int64_t id = t * TILE_ROWS + (wr * MR + b) * 32 + l32;
            inv_n[b] = invnorm[id < N ? id : N - 1];
        }
    };

    // Start of a tile.  The accumulators are not zeroed but initialised, by one MFMA per 32x32 block,
    // with  - threshold[query] * norm[row] : the filter  score * invnorm >= threshold  is
    // score - threshold * norm >= 0, so after the k-loop the epilogue only has to look at signs.
    // The operands are a 3-term extension, query side (th, th, tl), bank side -(nh, nl, nh), with
    // threshold = th + tl and norm = nh + nl in the operands' 16-bit type (the dropped tl*nl term and
    // the residuals are ~2^-16 relative, inside the margin).  The sparsest pass has no threshold: its
    // query-side extension is zero and the accumulators start at zero.
    auto tile_init = [&](int ti) __attribute__((always_inline)) {
#pragma unroll
        for (int b = 0; b < MR; ++b) inv_r[b] = inv_n[b];
        load_invnorm(ti + 1);
        uint32_t bx[MR], by[MR];
#pragma unroll
        for (int b = 0; b < MR; ++b) {
            const float norm = 1.0f / inv_r[b];
            const uint16_t nh = enc16(norm), nl = enc16(norm - dec16(nh));
            const uint32_t mh = nh ^ 0x8000u, ml = nl ^ 0x8000u;
            bx[b] = half ? 0u : (mh | (ml << 16));
            by[b] = half ? 0u : mh;
        }
        const bool use_thr = L.rho != 0;
#pragma unroll
        for (int a = 0; a < MQ; ++a) {
            const uint32_t tp = use_thr ? thp_s[(wq * MQ + a) * 32 + l32] : 0u;
            const u32x4_t aext = {half ? 0u : ((tp & 0xffffu) | (tp << 16)), half ? 0u : (tp >> 16), 0u, 0u};
#pragma unroll
            for (int b = 0; b < MR; ++b) {
                const u32x4_t bext = {bx[b], by[b], 0u, 0u};
                const f32x16_t z = {0.f};
                acc[a][b] = mfma32<DT == 0 ? 1 : DT>(aext, bext, z);
            }
        }
    };

    // ---- per-tile epilogue (all lanes of the workgroup call it together) ----
    auto epilogue = [&](int ti) __attribute__((always_inline)) {
        const int j = first_j + ti * stride_j;
        const int64_t t = level_tile(L, j);
        // The lane coordinates are re-derived from an opaque zero, so that the many per-lane output
        // addresses below are computed here, once per tile, instead of being hoisted out of the
        // k-loop and kept (spilled) across it.
        if (L.rho == 0) {
            // Sparsest pass: no threshold yet, every row is kept.  Slot = position of the row in
            // this pass, so no counter is needed (the count was preset to the pass's valid rows).
#pragma unroll
            for (int b = 0; b < MR; ++b) {
                int opaque = 0;
                asm volatile("" : "+v"(opaque));
                const int half = (lane >> 5) + opaque, l32 = (lane & 31) + opaque;
                const int rt = (wr * MR + b) * 32 + l32;
                const int64_t id = t * TILE_ROWS + rt;
                if (id < N) {
                    const float inve = inv_r[b];
                    const int64_t pos = (int64_t)j * TILE_ROWS + rt;
#pragma unroll
                    for (int a = 0; a < MQ; ++a) {
                        int opq = 0;
                        asm volatile("" : "+v"(opq));
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int ql = (wq * MQ + a) * 32 + 4 * (half + opq) + 8 * (r >> 2) + (r & 3);
                            surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = pack_key(acc[a][b][r] * inve * invq_s[ql], (int32_t)id);
                        }
                        __builtin_amdgcn_sched_barrier(0);
                    }
                }
            }
        } else {
            // Filter against the per-query thresholds.  Survivors (rare) go to a workgroup list in
            // LDS first, so that the global slot counters are bumped once per (workgroup, query)
            // and all at the same time, instead of one dependent device-wide atomic per survivor.
            // The accumulators hold  score - threshold * norm  (see tile_init): survivors are the
            // non-negative values.
            // Pass 1.  Float bit patterns compared as signed integers: negative floats are
            // negative integers, so "some value >= +0" is "integer max >= 0" (max3, no NaN handling).
            uint32_t msk[MQ * MR];
            uint32_t mine = 0;
#pragma unroll
            for (int b = 0; b < MR; ++b) {
                int opaque = 0;
                asm volatile("" : "+v"(opaque));
                const bool valid = t * TILE_ROWS + (wr * MR + b) * 32 + (lane & 31) + opaque < N;
#pragma unroll
                for (int a = 0; a < MQ; ++a) {
                    int mx = max((int)__float_as_uint(acc[a][b][0]), (int)__float_as_uint(acc[a][b][1]));
#pragma unroll
                    for (int r = 2; r < 16; r += 2)
                        mx = max(mx, max((int)__float_as_uint(acc[a][b][r]), (int)__float_as_uint(acc[a][b][r + 1])));
                    const bool hit = valid && mx >= 0;
                    uint32_t m = 0;
                    if (__builtin_amdgcn_ballot_w64(hit) != 0) {      // most blocks have no hit at all
                        uint32_t neg = 0;                                // sign bits, register 15 first
                        asm volatile("" : "+v"(neg));                   // keeps this a real branch
#pragma unroll
                        for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[a][b][r]), 31);
                        m = hit ? (~neg & 0xffffu) : 0u;
                    }
                    msk[a * MR + b] = m;
                    mine += __popc(m);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // Slots: a lane with survivors reserves them with one LDS atomic.
            if (__builtin_amdgcn_ballot_w64(mine != 0) != 0) {          // uniform within the wavefront
                uint32_t slot = mine ? atomicAdd(total_s, mine) : 0u;
                // Pass 2, survivors only.  Per block the union of the lanes' masks is brought into a
                // scalar (DPP or-reduction), and only the registers named by its bits are visited.
#pragma unroll
                for (int b = 0; b < MR; ++b) {
                    int opaque = 0;
                    asm volatile("" : "+v"(opaque));
                    const int half = (lane >> 5) + opaque, l32 = (lane & 31) + opaque;
                    const int32_t id = (int32_t)(t * TILE_ROWS + (wr * MR + b) * 32 + l32);
                    const float inve = inv_r[b];
                    const float norm = 1.0f / inve;
                    const float nh_v = dec16(enc16(norm)), nl_v = dec16(enc16(norm - nh_v));
#pragma unroll
                    for (int a = 0; a < MQ; ++a) {
                        const uint32_t m = msk[a * MR + b];
                        uint32_t wm = wave_or(m);                          // scalar
                        const int qb = (wq * MQ + a) * 32 + 4 * half;
                        while (wm) {
                            const int r = __builtin_ctz(wm);
                            wm &= wm - 1;
                            float av;
                            switch (r) {                                   // r is uniform: a scalar branch tree
                                case 0: av = acc[a][b][0]; break;   case 1: av = acc[a][b][1]; break;
                                case 2: av = acc[a][b][2]; break;   case 3: av = acc[a][b][3]; break;
                                case 4: av = acc[a][b][4]; break;   case 5: av = acc[a][b][5]; break;
                                case 6: av = acc[a][b][6]; break;   case 7: av = acc[a][b][7]; break;
                                case 8: av = acc[a][b][8]; break;   case 9: av = acc[a][b][9]; break;
                                case 10: av = acc[a][b][10]; break; case 11: av = acc[a][b][11]; break;
                                case 12: av = acc[a][b][12]; break; case 13: av = acc[a][b][13]; break;
                                case 14: av = acc[a][b][14]; break; default: av = acc[a][b][15]; break;
                            }
                            if (m & (1u << r)) {
                                const int ql = qb + 8 * (r >> 2) + (r & 3);
                                const uint32_t tp = thp_s[ql];
                                const float th = dec16((uint16_t)(tp & 0xffffu)), tl = dec16((uint16_t)(tp >> 16));
                                const float dot = av + (th * nh_v + th * nl_v + tl * nh_v);
                                const uint64_t key = pack_key(dot * inve * invq_s[ql], id);
                                if (slot < (uint32_t)SCAN_LIST_CAP) { lkey[slot] = key; lq[slot] = (uint32_t)ql; }
                                else {   // list full (a very loose threshold): fall back to the direct path
                                    uint32_t pos = atomicAdd(cnt + q0 + ql, 1u);
                                    if (pos < (uint32_t)SURV_CAP) surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = key;
                                }
                                ++slot;
                            }
                        }
                    }
                }
            }
            // The list is carried from tile to tile and written out every `flush_every` tiles (the host
            // sizes that from the expected number of survivors per tile; a surplus takes the direct
            // path above) and once at the end, so the device-wide round trip is paid every few tiles.
            if (ti % flush_every == flush_every - 1 || ti == my_tiles - 1) {     // uniform
                __syncthreads();
                flush();
            }
        }
    };

    // ---- pipeline over the flattened (tile, k-block) sequence; g counts steps over all tiles ----
    auto phase = [&](int s, u32x4_t (&gb)[BCH], u32x4_t (&gq)[QCH]) __attribute__((always_inline)) {
        // LDS stage s holds the current step; registers gb/gq hold the operands of the next one.  As
        // soon as those are in LDS (half-way through the MFMAs) the same registers take the loads of
        // the step three ahead, so two register sets are in flight at all times, tile epilogues included.
        compute(s, [&]() __attribute__((always_inline)) {
            lstore(s ^ 1, gb, gq);
            gload_q(gq);
            gload(gb);
        });
        __syncthreads();
    };
    gload_q(gqA);
    gload(gbA);
    gload_q(gqB);
    gload(gbB);
    lstore(0, gbA, gqA);
    gload_q(gqA);
    gload(gbA);
    __syncthreads();
    load_invnorm(0);
    for (int ti = 0; ti < my_tiles; ++ti) {
        tile_init(ti);
        for (int st = 0; st < nsteps; st += 2) {
            phase(0, gbB, gqB);
            phase(1, gbA, gqA);
        }
        epilogue(ti);
    }
}

}  // namespace evk
