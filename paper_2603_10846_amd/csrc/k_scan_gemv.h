// Similarity scan for small query batches over fp32 stores (Sec. 3.2, dense recall): a
// bandwidth-bound GEMV.
//
// At one to four queries the scan does 2*NB flops per element read, far below what the vector ALUs
// sustain per byte of HBM traffic: every lane streams 16-byte pieces of the tiled store and keeps NB
// running dot products per row in registers, in full fp32 (the matrix-core scan would have to split
// every fp32 value into two bf16 halves first, which is more vector work than the dot product).
// For 16-bit stores the same kernel shape was measured against the matrix-core scan run with a
// 32-query tile: 5.4-5.6 TB/s against 6.1 TB/s on a 1M x 1024 bf16 bank at one and at four queries
// (occupancy-driven, persistent with double-buffered registers, queries in LDS: all the same), so
// 16-bit stores use the matrix-core scan's load pipeline at every batch size.
//
// One workgroup (256 lanes) scans one 256-row tile.  16 lanes share a row (one 16-byte chunk of the
// row's k-block segment each), so one load instruction of the workgroup covers 16 rows x one
// k-block, and 16 such loads cover the tile; the partial sums of a row are combined with
// cross-lane adds at the end.  A similarity that reaches the query's current threshold (the k1-th
// best found by sparser passes, minus a rounding margin) is appended to the query's survivor list.
// A pass with few tiles (a small bank) gives each tile to four workgroups of 64 rows each, so that
// more compute units pull on the memory system: such a pass is bound by latency, not bandwidth.
#pragma once
#include "layout.h"

namespace evk {

__device__ __forceinline__ void append_survivor(float v, float invq_b, int32_t id, uint32_t* cnt_b,
                                                uint64_t* surv_b) {
    uint32_t pos = atomicAdd(cnt_b, 1u);           // integer slot counter; order is fixed later by sorting
    if (pos < (uint32_t)SURV_CAP) surv_b[pos] = pack_key(v * invq_b, id);
}

// fp32 stores: CH = 16 chunks of 4 elements per 256-byte segment.
// RG: groups of 16 rows a workgroup scans (16 = a whole tile; 4 = a quarter, gridDim.x = 4 * tiles).
template <int NB, int RG>
__global__ __launch_bounds__(256) void k_scan_gemv32(const float* __restrict__ store,
                                                     const float* __restrict__ invnorm,
                                                     const float* __restrict__ qf, const float* __restrict__ invq,
                                                     const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                     uint64_t* __restrict__ surv, int64_t N, int nkb, int B,
                                                     Level L, Mask mask) {
    const int tid = threadIdx.x, c = tid & 15, rbase = tid >> 4;   // rbase 0..15
    constexpr int PARTS = 16 / RG;
    const int tile_j = (int)blockIdx.x / PARTS, g0 = ((int)blockIdx.x % PARTS) * RG;   // first row group
    const int64_t t = level_tile(L, tile_j);
    const int dpad = nkb * KB;
    float acc[RG][NB];
#pragma unroll
    for (int i = 0; i < RG; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[i][b] = 0.f;
    const float* blk = store + t * nkb * (int64_t)BLOCK_ELEMS + (g0 * 16 + rbase) * KB + c * 4;
    for (int kb = 0; kb < nkb; ++kb, blk += BLOCK_ELEMS) {
        float4 x[RG];
#pragma unroll
        for (int i = 0; i < RG; ++i) x[i] = stream_load_float4(blk + i * 16 * KB);
        float4 qv[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
            qv[b] = *reinterpret_cast<const float4*>(qf + (int64_t)(b < B ? b : 0) * dpad + kb * KB + c * 4);
#pragma unroll
        for (int i = 0; i < RG; ++i)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float a = acc[i][b];
                a = fmaf(x[i].x, qv[b].x, a); a = fmaf(x[i].y, qv[b].y, a);
                a = fmaf(x[i].z, qv[b].z, a); a = fmaf(x[i].w, qv[b].w, a);
                acc[i][b] = a;
            }
    }
#pragma unroll
    for (int i = 0; i < RG; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = acc[i][b];
            v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64); v += __shfl_xor(v, 8, 64);
            acc[i][b] = v;
        }
#pragma unroll
    for (int i = 0; i < RG; ++i) {
        if (c != i) continue;
        int64_t id = t * TILE_ROWS + (g0 + i) * 16 + rbase;
        if (id >= N) continue;
        float inve = invnorm[id];
        const uint32_t tag = mask.tags ? mask.tags[id] : 0u;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b >= B) break;
            float v = acc[i][b] * inve;
            const bool ok = !mask.tags || eligible(tag, mask.allow[b], mask.exclude[b]);
            if (L.rho == 0)      // sparsest pass keeps every row at its own position, no counter (0 = empty slot)
                surv[(int64_t)b * SURV_CAP + (int64_t)tile_j * TILE_ROWS + (id - t * TILE_ROWS)] = ok ? pack_key(v * invq[b], (int32_t)id) : 0ull;
            else if (ok && v >= thr[b]) append_survivor(v, invq[b], (int32_t)id, cnt + b, surv + (int64_t)b * SURV_CAP);
        }
    }
}

}  // namespace evk
