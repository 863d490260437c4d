// Similarity scan on the matrix cores (Sec. 3.2, dense recall): scores[q][n] = <query q, bank row n>,
// never written to memory.  Used for every batch size on 16-bit stores (at a handful of queries the
// arithmetic is idle and the kernel is a streaming engine for the bank) and for more than four
// queries on fp32 stores.
//
// Persistent workgroups of 4 or 8 wavefronts; each owns QT queries and walks over 256-row bank
// tiles.  Per k-block the bank tile's 32 KB block (already in LDS operand order in HBM, see
// layout.h) and the queries' block are staged in LDS (two stages) and consumed by
// v_mfma_f32_32x32x16 (bf16 or f16 operands, fp32 accumulation).  Global loads run two k-blocks
// ahead of the MFMAs through two register sets, and the (tile, k-block) sequence is flattened, so
// the loads of the next tile are already in flight while a tile's epilogue runs.  Queries are the
// rows of the accumulator tile and bank rows its columns: a lane holds one bank row per 32x32 block.
// Within a k-block the four k-steps are a hand-written software pipeline (see compute()): operand
// fragments are read from LDS one k-step ahead, the LDS stores and global loads of the following
// k-blocks issue between the MFMAs, and there is one workgroup barrier per k-block.
//
// fp32 stores: each value is split on the fly into bf16 hi + bf16 lo and the product is
// hi*hi + hi*lo + lo*hi (three MFMAs, relative error of a product about 2^-16); this only has to
// be good enough for the filter, since the value filter re-scores the selected candidates in fp64.
//
// Filter: the accumulators of a tile start at  -threshold[query] * norm[row]  (one extra MFMA per
// block), so after the k-loop a score passes iff its accumulator is non-negative; the epilogue
// collects sign bits, stages the rare survivors in an LDS list and flushes it every few tiles.
// The sparsest pass has no threshold and writes every row's key to the row's own position.
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

// Two fp32 values rounded to bf16 (round to nearest even) and packed, a first: one v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
    typedef __attribute__((ext_vector_type(2))) float f32x2_t;
    typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// hi/lo split of two fp32 values for the matrix cores: returns the packed bf16 heads and leaves the
// (exactly representable) remainders a - head(a), b - head(b) in ra, rb.
__device__ __forceinline__ uint32_t pack_bf16x2_hi(float a, float b, float& ra, float& rb) {
    const uint32_t h = cvt_pk_bf16(a, b);
    ra = a - __uint_as_float(h << 16);
    rb = b - __uint_as_float(h & 0xffff0000u);
    return h;
}

// Per-lane choice of one of the 16 registers of an accumulator block: register r = 4 * hi + lo of each
// lane's own (lo, hi), given as lane masks (lo == 1, lo == 3, lo >= 2, hi == 1, hi == 3, hi >= 2).  A
// two-level tree of 15 v_cndmask (registers cannot be indexed per lane).  Written as instructions because
// the compiler turns the equivalent C++ selects over elements of an accumulator vector into a
// dynamically indexed vector access, which it expands to a 16-way chain.  The two wait states at the
// top are the ones gfx950 needs between a vector compare writing a mask and a vector instruction reading
// it; the compiler does not add them for instructions it cannot see, and one pair serves all 15.
__device__ __forceinline__ float lane_select16(const f32x16_t& v, uint64_t lo1, uint64_t lo3, uint64_t lo23,
                                               uint64_t hi1, uint64_t hi3, uint64_t hi23) {
    float g0, g1, g2, g3, t;
    asm("s_nop 1\n\t"
        "v_cndmask_b32_e64 %[g0], %[a0], %[a1], %[lo1]\n\t"
        "v_cndmask_b32_e64 %[t], %[a2], %[a3], %[lo3]\n\t"
        "v_cndmask_b32_e64 %[g0], %[g0], %[t], %[lo23]\n\t"
        "v_cndmask_b32_e64 %[g1], %[a4], %[a5], %[lo1]\n\t"
        "v_cndmask_b32_e64 %[t], %[a6], %[a7], %[lo3]\n\t"
        "v_cndmask_b32_e64 %[g1], %[g1], %[t], %[lo23]\n\t"
        "v_cndmask_b32_e64 %[g2], %[a8], %[a9], %[lo1]\n\t"
        "v_cndmask_b32_e64 %[t], %[a10], %[a11], %[lo3]\n\t"
        "v_cndmask_b32_e64 %[g2], %[g2], %[t], %[lo23]\n\t"
        "v_cndmask_b32_e64 %[g3], %[a12], %[a13], %[lo1]\n\t"
        "v_cndmask_b32_e64 %[t], %[a14], %[a15], %[lo3]\n\t"
        "v_cndmask_b32_e64 %[g3], %[g3], %[t], %[lo23]\n\t"
        "v_cndmask_b32_e64 %[g0], %[g0], %[g1], %[hi1]\n\t"
        "v_cndmask_b32_e64 %[g2], %[g2], %[g3], %[hi3]\n\t"
        "v_cndmask_b32_e64 %[g0], %[g0], %[g2], %[hi23]"
        : [g0] "=&v"(g0), [g1] "=&v"(g1), [g2] "=&v"(g2), [g3] "=&v"(g3), [t] "=&v"(t)
        : [a0] "v"(v[0]), [a1] "v"(v[1]), [a2] "v"(v[2]), [a3] "v"(v[3]), [a4] "v"(v[4]), [a5] "v"(v[5]), [a6] "v"(v[6]),
          [a7] "v"(v[7]), [a8] "v"(v[8]), [a9] "v"(v[9]), [a10] "v"(v[10]), [a11] "v"(v[11]), [a12] "v"(v[12]),
          [a13] "v"(v[13]), [a14] "v"(v[14]), [a15] "v"(v[15]), [lo1] "s"(lo1), [lo3] "s"(lo3), [lo23] "s"(lo23),
          [hi1] "s"(hi1), [hi3] "s"(hi3), [hi23] "s"(hi23));
    return g0;
}

// The one non-negative value among the 16 registers of an accumulator block, for lanes that have exactly
// one: as signed integers, every value with the sign bit set is below every value without it, so the
// integer maximum of the bit patterns is that value, bit for bit (8 three-operand maxima; no compare
// masks and no per-lane register choice).
__device__ __forceinline__ float only_non_negative(const f32x16_t& v) {
    auto bits = [&](int r) __attribute__((always_inline)) { return (int)__float_as_uint(v[r]); };
    auto max3 = [](int a, int b, int c) __attribute__((always_inline)) { return max(max(a, b), c); };
    const int t0 = max3(bits(0), bits(1), bits(2)), t1 = max3(bits(3), bits(4), bits(5)), t2 = max3(bits(6), bits(7), bits(8));
    const int t3 = max3(bits(9), bits(10), bits(11)), t4 = max3(bits(12), bits(13), bits(14));
    return __uint_as_float((uint32_t)max(max3(t0, t1, t2), max3(t3, t4, bits(15))));
}

// Inclusive prefix sum over the 64 lanes of a wavefront (all lanes active): shifts within rows of 16
// lanes, then the row broadcasts.  Lane 63 ends up with the total.
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x) {
    int v = (int)x;
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, true);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, true);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, true);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, true);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, true);   // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, true);   // row_bcast:31 into rows 2 and 3
    return (uint32_t)v;
}

constexpr int STAGE_BANK_BYTES = TILE_ROWS * 128;
constexpr int SCAN_LIST_CAP = 2048;     // survivor entries a workgroup can stage per tile

// LDS: two stages (bank tile + query tile); per-query threshold, inverse norm, survivor count and
// list base; the workgroup's survivor list (8-byte key + 4-byte query index per entry); a counter.
// (masked variant: the per-query type masks and excluded groups in addition)
template <int QT, bool MASKED = false> constexpr int scan_mfma_lds_bytes() {
    return 2 * (STAGE_BANK_BYTES + QT * 128) + QT * 16 + SCAN_LIST_CAP * 12 + 16 + (MASKED ? QT * 8 : 0);
}

// DT: 0 fp32 store (bf16 split), 1 bf16, 2 f16.  Wave grid WQ x WR, each wave MQ x MR blocks of 32x32.
// gridDim.x is a multiple of 8 * (Bp / QT).
// MASKED: typed / masked retrieval -- a row is kept for a query only if the query accepts its tag.
// STREAM: bank rows are loaded with the non-temporal hint (layout.h).  Right whenever a bank tile is read
// by one workgroup only; with several query tiles per bank tile (more than 256 queries) the later readers
// are meant to find the tile in L2, and the hint costs 7 % there (measured: 1185 -> 1105 TFLOP/s at 1024 queries).
template <int DT, int MQ, int WQ, int MR, int WR, bool MASKED, bool STREAM = true>
__global__ __launch_bounds__(64 * WQ * WR) void k_scan_mfma(const void* __restrict__ store_, const float* __restrict__ invnorm,
                                                   const uint16_t* __restrict__ qop, const float* __restrict__ invq,
                                                   const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                   uint64_t* __restrict__ surv, int64_t N, int nkb, int Bp,
                                                   Level L, int flush_every, Mask mask, int B) {
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
    // Outside the k-loop (tile start, epilogue) lane coordinates are formed afresh: the wavefront's
    // position from scalar registers, the lane index from the lane counter seeded with a zero the
    // compiler cannot see through.  A per-lane value kept from the kernel's start would live on the
    // stack across the k-loop (there is no register to spare), and the wait for its reload is a wait
    // for every load in flight.
    const int wq_u = __builtin_amdgcn_readfirstlane(wq), wr_u = __builtin_amdgcn_readfirstlane(wr);
    auto fresh_lane = [&]() __attribute__((always_inline)) {
        uint32_t z = 0;
        asm volatile("" : "+v"(z));
        return (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, z));
    };

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
    constexpr uint32_t LKEY_OFF = 2 * STAGE_BYTES + QT * 16, LQ_OFF = LKEY_OFF + SCAN_LIST_CAP * 8;   // the list's two arrays
    uint64_t* lkey = reinterpret_cast<uint64_t*>(smem + LKEY_OFF);
    uint32_t* lq = reinterpret_cast<uint32_t*>(smem + LQ_OFF);
    uint32_t* total_s = lq + SCAN_LIST_CAP;
    uint32_t* allow_s = total_s + 4;                    // masked variant only
    uint32_t* exclude_s = allow_s + QT;
    for (int i = tid; i < QT; i += NT) {
        const float th = thr[q0 + i];
        const uint16_t hi = enc16(th), lo = enc16(th - dec16(hi));
        thp_s[i] = hi | ((uint32_t)lo << 16);
        invq_s[i] = invq[q0 + i];
        cnt_s[i] = 0;
        if constexpr (MASKED) {                         // padding queries accept nothing
            allow_s[i] = q0 + i < B ? mask.allow[q0 + i] : 0u;
            exclude_s[i] = q0 + i < B ? mask.exclude[q0 + i] : 0u;
        }
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
    // (the cursor step and the loads themselves are separate, so that the loads can be issued one
    // at a time between MFMAs)
    auto gnext_q = [&]() __attribute__((always_inline)) {
        const uint16_t* qb = qop + ((int64_t)rotated(ldq_step) * Bp + q0) * KB;
        if (++ldq_step == nsteps) ldq_step = 0;
        return qb;
    };
    auto gpiece = [&](const uint16_t* base, int i) __attribute__((always_inline)) {
        return *reinterpret_cast<const u32x4_t*>(base + (i * NT + tid) * 8);
    };
    auto gpiece_bank = [&](const uint16_t* base, int i) __attribute__((always_inline)) {
        if constexpr (STREAM) return __builtin_bit_cast(u32x4_t, stream_load16(base + (i * NT + tid) * 8));
        else return *reinterpret_cast<const u32x4_t*>(base + (i * NT + tid) * 8);
    };
    auto gload_q = [&](u32x4_t (&gq)[QCH]) __attribute__((always_inline)) {
        const uint16_t* qb = gnext_q();
#pragma unroll
        for (int i = 0; i < QCH; ++i) gq[i] = gpiece(qb, i);
    };
    // first element of the bank tile the load cursor is on (recomputed only when the cursor moves on
    // to another tile: level_tile() contains an integer division)
    int64_t ld_tile_elem = level_tile(L, first_j) * nkb * (int64_t)BLOCK_ELEMS;
    auto gnext_b = [&]() __attribute__((always_inline)) {     // 16-bit stores only
        const int kb = ld_step < real_steps ? rotated(ld_step) : real_steps - 1;
        const uint16_t* blk = static_cast<const uint16_t*>(store_) + ld_tile_elem + kb * (int64_t)BLOCK_ELEMS;
        if (++ld_step == nsteps) {
            ld_step = 0;
            if (ld_ti + 1 < my_tiles) { ++ld_ti; ld_tile_elem = level_tile(L, first_j + ld_ti * stride_j) * nkb * (int64_t)BLOCK_ELEMS; }
        }
        return blk;
    };
    auto gload = [&](u32x4_t (&gb)[BCH]) __attribute__((always_inline)) {
        if constexpr (DT == 0) {
            const float* blk = static_cast<const float*>(store_) + ld_tile_elem + (rotated(ld_step) >> 1) * (int64_t)BLOCK_ELEMS + (rotated(ld_step) & 1) * 32;
#pragma unroll
            for (int i = 0; i < BCH; ++i) {
                int g = i * NT + tid, r = g >> 3, c4 = g & 7;
                if constexpr (STREAM) gb[i] = __builtin_bit_cast(u32x4_t, stream_load16(blk + r * KB + c4 * 4));
                else gb[i] = *reinterpret_cast<const u32x4_t*>(blk + r * KB + c4 * 4);
            }
            // past the last step the cursor stays on the last tile: the loads issued there are never
            // consumed, but keeping every step free of branches lets the loads stay in flight across it
            if (++ld_step == nsteps) {
                ld_step = 0;
                if (ld_ti + 1 < my_tiles) { ++ld_ti; ld_tile_elem = level_tile(L, first_j + ld_ti * stride_j) * nkb * (int64_t)BLOCK_ELEMS; }
            }
        } else {
            const uint16_t* blk = gnext_b();
#pragma unroll
            for (int i = 0; i < BCH; ++i) gb[i] = gpiece_bank(blk, i);
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
                lo.x = cvt_pk_bf16(r0, r1);
                lo.y = cvt_pk_bf16(r2, r3);
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
    // The k-step enters through bits 5..6 only, so the address for k-step k4 is the one for k-step 0
    // with (k4 << 5) xor-ed in: one per-lane offset per operand (the wave's first block folded in)
    // serves every block, both stages and all k-steps; the rest is a compile-time constant.
    const uint32_t off0 = l32 * 128 + swz16(half, l32) * 16;
    const uint32_t offA0 = off0 + STAGE_BANK_BYTES + wq * MQ * 4096, offB0 = off0 + wr * MR * 4096;
    uint32_t offA[4], offB[4];
#pragma unroll
    for (int k4 = 0; k4 < 4; ++k4) { offA[k4] = offA0 ^ (k4 << 5); offB[k4] = offB0 ^ (k4 << 5); }
    auto frag = [&](int s, uint32_t off, int block) __attribute__((always_inline)) {
        return *reinterpret_cast<const u32x4_t*>(smem + off + (s * STAGE_BYTES + block * 4096));
    };
    // One step: the MFMAs on LDS stage s, and meanwhile the operands of the next step (registers gb, gq,
    // loaded two steps ago) go to stage s ^ 1 and the same registers take the loads of the step three
    // ahead, so two register sets are in flight at all times, tile epilogues included.
    // Inverse norms of this lane's MR bank rows of the next tile.  They are requested in the last
    // k-step of a tile (the fragment registers are free by then; across the whole k-loop there is
    // no register to spare, and a value that gets spilled has to be waited for right after its
    // request, which drains every load in flight) and turned into MFMA operands (tile_prepare)
    // after that tile's epilogue, by when they have long arrived.  The rare epilogue paths that
    // need an inverse norm of the current tile read it from memory again.
    float inv_n[MR];
    int tile_now = 0;
    auto load_invnorm = [&](int ti) __attribute__((always_inline)) {
        const int64_t t = level_tile(L, first_j + (ti < my_tiles ? ti : my_tiles - 1) * stride_j);
        const int row0 = (wr_u * MR) * 32 + (fresh_lane() & 31);
#pragma unroll
        for (int b = 0; b < MR; ++b) {
            const int64_t id = t * TILE_ROWS + row0 + b * 32;
            inv_n[b] = invnorm[id < N ? id : N - 1];
        }
    };

    u32x4_t af[MQ], bfr[2][MR];   // operand fragments of the 16-bit path, carried from step to step
    auto compute = [&](int s, u32x4_t (&gb)[BCH], u32x4_t (&gq)[QCH], auto fetch_next) __attribute__((always_inline)) {
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
                if (ks == 0) {
                    lstore(s ^ 1, gb, gq);
                    gload_q(gq);
                    gload(gb);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        } else {
            // A software pipeline written out by hand, one slot per query block a of a k-step:
            //   the MFMAs of block a (MR of them), then the LDS read of block a's fragment for the next
            //   k-step into the registers those MFMAs have just read, then one piece of the side work.
            // The bank fragments are used by every slot and are double buffered instead.  So every
            // fragment is requested at least MR * (MQ - 1) MFMAs before its first use and a wavefront
            // can keep the matrix pipe busy by itself; the LDS stores (k-steps 1 and 2) and the global
            // loads (k-step 3) issue in the shadow of the MFMAs instead of forming a period without any.
            // The scheduler is fenced per slot to keep this order (left alone it hoists the reads).
            // On entry af and bfr[0] hold the fragments of k-step 0, fetched by the previous step or, for
            // the first step of a tile, by the tile loop (the last step of a tile fetches nothing: the
            // fragments would only occupy registers that the tile epilogue needs).
            constexpr bool FETCH = decltype(fetch_next)::value;
            const uint16_t* nq = gnext_q();
            const uint16_t* nb = gnext_b();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                const int cur = ks & 1;
                const uint32_t oa = offA0 ^ (((ks + 1) & 3) << 5), ob = offB0 ^ (((ks + 1) & 3) << 5);
                // The step's only barrier: every wavefront has stored its share of stage s ^ 1 (k-steps
                // 1 and 2) and has received all it reads from stage s (the fragments of k-step 3 were
                // requested during k-step 2).  After it, k-step 3 still has its operands in registers,
                // and its slots fetch the first fragments of the next step from stage s ^ 1, so the
                // matrix pipe does not wait for LDS after the barrier.
                if (ks == 3) __syncthreads();
                if (ks < 3 || FETCH) {
#pragma unroll
                    for (int b = 0; b < MR; ++b) bfr[cur ^ 1][b] = frag(ks < 3 ? s : s ^ 1, ob, b);
                }
#pragma unroll
                for (int a = 0; a < MQ; ++a) {
#pragma unroll
                    for (int b = 0; b < MR; ++b) acc[a][b] = mfma32<DT>(af[a], bfr[cur][b], acc[a][b]);
                    if (ks < 3 || FETCH) af[a] = frag(ks < 3 ? s : s ^ 1, oa, a);
                    if (ks == 1) {
#pragma unroll
                        for (int i = a * QCH / MQ; i < (a + 1) * QCH / MQ; ++i)
                            *reinterpret_cast<u32x4_t*>(sq(s ^ 1) + (i * NT + tid) * 16) = gq[i];
                    }
                    if (ks == 2) {
#pragma unroll
                        for (int i = a * BCH / MQ; i < (a + 1) * BCH / MQ; ++i)
                            *reinterpret_cast<u32x4_t*>(sbank(s ^ 1) + (i * NT + tid) * 16) = gb[i];
                    }
                    // the registers stored during k-step 1 (query pieces) are reloaded during k-step 2,
                    // those stored during k-step 2 (bank pieces) during k-step 3, a few per slot
                    if (ks == 2) {
#pragma unroll
                        for (int i = a * QCH / MQ; i < (a + 1) * QCH / MQ; ++i) gq[i] = gpiece(nq, i);
                    }
                    if (ks == 3) {
#pragma unroll
                        for (int i = a * BCH / MQ; i < (a + 1) * BCH / MQ; ++i) gb[i] = gpiece_bank(nb, i);
                        if (!FETCH && a == MQ - 1) load_invnorm(tile_now + 1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
    };

    // Key of a survivor from its accumulator value (score - threshold * norm, see tile_init): the
    // threshold term is added back exactly as the MFMA formed it, then the cosine is taken.
    auto finish_key = [&](float av, int ql, int32_t id, float inv) __attribute__((always_inline)) {
        const float norm = __builtin_amdgcn_rcpf(inv);
        const float nh = dec16(enc16(norm)), nl = dec16(enc16(norm - nh));
        const uint32_t tp = thp_s[ql];
        const float th = dec16((uint16_t)(tp & 0xffffu)), tl = dec16((uint16_t)(tp >> 16));
        const float dot = av + (th * nh + th * nl + tl * nh);
        return pack_key(dot * inv * invq_s[ql], id);
    };

    // Write the workgroup's staged survivors to the per-query lists (all lanes call it together):
    // rank the entries of each query with LDS atomics, reserve that many slots with one device-wide
    // integer atomic per query that has any, copy.
    auto flush = [&]() __attribute__((always_inline)) {
        const uint32_t total = *total_s < (uint32_t)SCAN_LIST_CAP ? *total_s : (uint32_t)SCAN_LIST_CAP;
        for (uint32_t e = tid; e < total; e += NT) {
            uint32_t ql = lq[e];
            if (MASKED && ql == 0xffffu) continue;            // a survivor its query does not accept
            lq[e] = ql | (atomicAdd(cnt_s + ql, 1u) << 16);   // rank among the staged entries of ql
        }
        __syncthreads();
        for (int i = tid; i < QT; i += NT) {
            uint32_t c = cnt_s[i];
            base_s[i] = c ? atomicAdd(cnt + q0 + i, c) : 0u;
            cnt_s[i] = 0;
        }
        __syncthreads();
        // four entries per lane at a time, so that their inverse-norm reads are in flight together
        for (uint32_t e0 = tid; e0 < total; e0 += 4 * NT) {
            float inv[4];
            uint64_t ent[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = e0 + k * NT;
                ent[k] = lkey[e < total ? e : e0];
                inv[k] = invnorm[(int32_t)(uint32_t)ent[k]];
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t e = e0 + k * NT;
                if (e < total && !(MASKED && (lq[e] & 0xffffu) == 0xffffu)) {
                    const uint32_t ql = lq[e] & 0xffffu, rank = lq[e] >> 16;
                    const uint32_t pos = base_s[ql] + rank;
                    if (pos < (uint32_t)SURV_CAP)
                        surv[(int64_t)(q0 + ql) * SURV_CAP + pos] =
                            finish_key(__uint_as_float((uint32_t)(ent[k] >> 32)), (int)ql, (int32_t)(uint32_t)ent[k], inv[k]);
                }
            }
        }
        __syncthreads();
        if (tid == 0) *total_s = 0;
        __syncthreads();
    };

    // Start of a tile.  The accumulators are not zeroed but initialised, by one MFMA per 32x32 block,
    // with  - threshold[query] * norm[row] : the filter  score * invnorm >= threshold  is
    // score - threshold * norm >= 0, so after the k-loop the epilogue only has to look at signs.
    // The operands are a 3-term extension, query side (th, th, tl), bank side -(nh, nl, nh), with
    // threshold = th + tl and norm = nh + nl in the operands' 16-bit type (the dropped tl*nl term and
    // the residuals are ~2^-16 relative, inside the margin).  The sparsest pass has no threshold: its
    // query-side extension is zero and the accumulators start at zero.
    // Norm operands of the tile about to start, from the inverse norms requested a tile earlier.
    uint32_t bx[MR], by[MR];
    auto tile_prepare = [&]() __attribute__((always_inline)) {
        const int half = fresh_lane() >> 5;
#pragma unroll
        for (int b = 0; b < MR; ++b) {
            const float norm = __builtin_amdgcn_rcpf(inv_n[b]);   // finish_key() forms it the same way
            const uint16_t nh = enc16(norm), nl = enc16(norm - dec16(nh));
            const uint32_t mh = nh ^ 0x8000u, ml = nl ^ 0x8000u;
            bx[b] = half ? 0u : (mh | (ml << 16));
            by[b] = half ? 0u : mh;
        }
    };
    auto tile_init = [&](int ti) __attribute__((always_inline)) {
        const bool use_thr = L.rho != 0;
        const int ln = fresh_lane(), half = ln >> 5, l32 = ln & 31;
#pragma unroll
        for (int a = 0; a < MQ; ++a) {
            const uint32_t tp = use_thr ? thp_s[(wq_u * MQ + a) * 32 + l32] : 0u;
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
        if (L.rho == 0) {
            // Sparsest pass: no threshold yet, every row is kept.  Slot = position of the row in
            // this pass, so no counter is needed (the count was preset to the pass's valid rows).
#pragma unroll
            for (int b = 0; b < MR; ++b) {
                const int ln = fresh_lane(), half = ln >> 5, l32 = ln & 31;
                const int rt = (wr_u * MR + b) * 32 + l32;
                const int64_t id = t * TILE_ROWS + rt;
                if (id < N) {
                    const float inve = invnorm[id];
                    uint32_t tag = 0;
                    if constexpr (MASKED) tag = mask.tags[id];
                    const int64_t pos = (int64_t)j * TILE_ROWS + rt;
#pragma unroll
                    for (int a = 0; a < MQ; ++a) {
                        int opq = 0;
                        asm volatile("" : "+v"(opq));
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int ql = (wq_u * MQ + a) * 32 + 4 * (half + opq) + 8 * (r >> 2) + (r & 3);
                            const bool ok = !MASKED || eligible(tag, allow_s[ql], exclude_s[ql]);
                            surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = ok ? pack_key(acc[a][b][r] * inve * invq_s[ql], (int32_t)id) : 0ull;   // 0 = empty slot
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
            // Pass 1.  Per block and lane a 16-bit mask of the non-negative accumulators, built from the
            // sign bits with one funnel shift per register (no test for "no survivor in this block"
            // first: at the survivor rates of the dense passes nearly every block has some).
            uint32_t msk[MQ * MR];
            uint32_t mine = 0;
#pragma unroll
            for (int b = 0; b < MR; ++b) {
                const bool valid = t * TILE_ROWS + (wr_u * MR + b) * 32 + (fresh_lane() & 31) < N;
#pragma unroll
                for (int a = 0; a < MQ; ++a) {
                    uint32_t neg = 0;                                    // sign bits, register 15 first
#pragma unroll
                    for (int r = 15; r >= 0; --r) neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(acc[a][b][r]), 31);
                    const uint32_t m = valid ? (~neg & 0xffffu) : 0u;
                    msk[a * MR + b] = m;
                    mine += __popc(m);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            // Slots: a prefix sum over the wavefront, one LDS atomic per wavefront for its total.
            if (__builtin_amdgcn_ballot_w64(mine != 0) != 0) {          // uniform within the wavefront
                const uint32_t incl = wave_inclusive_sum(mine);
                uint32_t wave_base = 0;
                if (fresh_lane() == 63) wave_base = atomicAdd(total_s, incl);
                uint32_t slot = (uint32_t)__builtin_amdgcn_readlane((int)wave_base, 63) + incl - mine;
                // Pass 2, survivors only, all lanes in parallel: each lane takes the first set bit of its
                // own mask, fetches that accumulator register with a two-level select (registers cannot
                // be indexed per lane) and stages (value, row id, query); the key is finished when the
                // list is flushed.  The first round over the blocks is straight-line code, so that the
                // blocks' instructions interleave; lanes that hold a second survivor of one block (few)
                // are served by a loop afterwards.
                auto pick = [&](int a, int b, int r) __attribute__((always_inline)) {
                    const int lo = r & 3, hi = (r >> 2) & 3;
                    return lane_select16(acc[a][b], __builtin_amdgcn_ballot_w64(lo == 1), __builtin_amdgcn_ballot_w64(lo == 3),
                                         __builtin_amdgcn_ballot_w64(lo >= 2), __builtin_amdgcn_ballot_w64(hi == 1),
                                         __builtin_amdgcn_ballot_w64(hi == 3), __builtin_amdgcn_ballot_w64(hi >= 2));
                };
                auto stage_one = [&](int a, int b, int r, float av) __attribute__((always_inline)) {   // lanes with a survivor
                    const int ln = fresh_lane(), half = ln >> 5, l32 = ln & 31;
                    const int32_t id = (int32_t)(t * TILE_ROWS + (wr_u * MR + b) * 32 + l32);
                    const int ql = (wq_u * MQ + a) * 32 + 4 * half + 8 * ((r >> 2) & 3) + (r & 3);
                    bool ok = true;
                    if constexpr (MASKED) ok = eligible(mask.tags[id], allow_s[ql], exclude_s[ql]);
                    if (slot < (uint32_t)SCAN_LIST_CAP) {
                        lkey[slot] = ((uint64_t)__float_as_uint(av) << 32) | (uint32_t)id;
                        lq[slot] = ok ? (uint32_t)ql : 0xffffu;          // the slot was reserved before the check
                    } else if (ok) {   // list full (a very loose threshold): fall back to the direct path
                        uint32_t pos = atomicAdd(cnt + q0 + ql, 1u);
                        if (pos < (uint32_t)SURV_CAP) surv[(int64_t)(q0 + ql) * SURV_CAP + pos] = finish_key(av, ql, id, invnorm[id]);
                    }
                    ++slot;
                };
                // First round, the common case kept free of inner branches: lanes with exactly one survivor in
                // a block stage it; lanes with more are left to the loop below, and so is everything when the
                // wavefront's reservation does not fit the list (then no lane needs a room check here).
                uint32_t rest = 0;
                const bool fits = (uint32_t)__builtin_amdgcn_readlane((int)wave_base, 63) + (uint32_t)__builtin_amdgcn_readlane((int)incl, 63)
                                  <= (uint32_t)SCAN_LIST_CAP;                                  // uniform
                const int ln0 = fresh_lane();
                const int32_t id0 = (int32_t)(t * TILE_ROWS + wr_u * MR * 32 + (ln0 & 31));   // this lane's row in block b = 0
                int qla[MQ];                                                                   // this lane's first query in block a
#pragma unroll
                for (int a = 0; a < MQ; ++a) qla[a] = (wq_u * MQ + a) * 32 + 4 * (ln0 >> 5);
                // running LDS addresses of the lane's next list entry (key array, query array)
                unsigned char* pk = smem + LKEY_OFF + slot * 8u;
                unsigned char* pq = smem + LQ_OFF + slot * 4u;
#pragma unroll
                for (int b = 0; b < MR; ++b)
#pragma unroll
                    for (int a = 0; a < MQ; ++a) {
                        const uint32_t m = msk[a * MR + b];
                        const bool take = fits && __popc(m) == 1;
                        if (take) {
                            const int r = __builtin_ctz(m);
                            const float av = only_non_negative(acc[a][b]);
                            const int32_t id = id0 + b * 32;
                            const int ql = qla[a] + r + (r & 12);            // register r holds query 8 * (r >> 2) + (r & 3) of the block
                            bool ok = true;
                            if constexpr (MASKED) ok = eligible(mask.tags[id], allow_s[ql], exclude_s[ql]);
                            *reinterpret_cast<uint64_t*>(pk) = ((uint64_t)__float_as_uint(av) << 32) | (uint32_t)id;
                            *reinterpret_cast<uint32_t*>(pq) = ok ? (uint32_t)ql : 0xffffu;   // the slot was reserved before the check
                            pk += 8;
                            pq += 4;
                        }
                        const uint32_t left = take ? 0u : m;
                        msk[a * MR + b] = left;
                        rest |= left;
                    }
                slot = (uint32_t)(pq - (smem + LQ_OFF)) >> 2;
                if (__builtin_amdgcn_ballot_w64(rest != 0) != 0) {
#pragma unroll
                    for (int b = 0; b < MR; ++b)
#pragma unroll
                        for (int a = 0; a < MQ; ++a) {
                            uint32_t m = msk[a * MR + b];
                            while (__builtin_amdgcn_ballot_w64(m != 0) != 0) {
                                const int r = __builtin_ctz(m | 0x10000u);
                                const float av = pick(a, b, r);
                                if (m) stage_one(a, b, r, av);
                                m &= m - 1;
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
    auto phase = [&](int s, u32x4_t (&gb)[BCH], u32x4_t (&gq)[QCH], auto fetch_next) __attribute__((always_inline)) {
        compute(s, gb, gq, fetch_next);
        if constexpr (DT == 0) __syncthreads();
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
    tile_prepare();
    for (int ti = 0; ti < my_tiles; ++ti) {
        tile_init(ti);
        tile_now = ti;
        if constexpr (DT == 0) load_invnorm(ti + 1);
        if constexpr (DT != 0) {
#pragma unroll
            for (int a = 0; a < MQ; ++a) af[a] = frag(0, offA0, a);
#pragma unroll
            for (int b = 0; b < MR; ++b) bfr[0][b] = frag(0, offB0, b);
        }
        for (int st = 0; st < nsteps - 2; st += 2) {
            phase(0, gbB, gqB, std::true_type{});
            phase(1, gbA, gqA, std::true_type{});
        }
        phase(0, gbB, gqB, std::true_type{});
        phase(1, gbA, gqA, std::false_type{});
        epilogue(ti);
        tile_prepare();
    }
}

}  // namespace evk
