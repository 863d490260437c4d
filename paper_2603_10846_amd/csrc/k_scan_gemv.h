// Similarity scan for small query batches (Sec. 3.2, dense recall): a bandwidth-bound GEMV.
//
// At one to four queries the scan does 2*NB flops per element read, far below what the vector ALUs
// sustain per byte of HBM traffic, so matrix cores would add nothing: every lane streams 16-byte
// pieces of the tiled store and keeps NB running dot products per row in registers.
//
// One workgroup (256 lanes) scans one 256-row tile.  CH lanes share a row (one 16-byte chunk of the
// row's k-block segment each), so one load instruction of the workgroup covers 256/CH rows x one
// k-block, and CH such loads cover the tile; the CH partial sums of a row are combined with
// cross-lane adds at the end.  A similarity that reaches the query's current threshold (the k1-th
// best found by sparser passes, minus a rounding margin) is appended to the query's survivor list.
#pragma once
#include "layout.h"

namespace evk {

__device__ __forceinline__ void append_survivor(float v, float invq_b, int32_t id, uint32_t* cnt_b,
                                                uint64_t* surv_b) {
    uint32_t pos = atomicAdd(cnt_b, 1u);           // integer slot counter; order is fixed later by sorting
    if (pos < (uint32_t)SURV_CAP) surv_b[pos] = pack_key(v * invq_b, id);
}

// 16-bit stores: CH = 8 chunks of 8 elements per 128-byte segment.
template <typename ST, int NB>
__global__ __launch_bounds__(256) void k_scan_gemv16(const uint16_t* __restrict__ store,
                                                     const float* __restrict__ invnorm,
                                                     const float* __restrict__ qf, const float* __restrict__ invq,
                                                     const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                     uint64_t* __restrict__ surv, int64_t N, int nkb, int B,
                                                     Level L, Mask mask) {
    const int tid = threadIdx.x, c = tid & 7, rbase = tid >> 3;   // rbase 0..31
    const int64_t t = level_tile(L, blockIdx.x);
    const int dpad = nkb * KB;
    float acc[8][NB];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[i][b] = 0.f;
    int poff[8];                                   // element offset of this lane's chunk in row group i
#pragma unroll
    for (int i = 0; i < 8; ++i) { int r = i * 32 + rbase; poff[i] = r * KB + swz16(c, r) * 8; }

    const uint16_t* blk = store + t * nkb * (int64_t)BLOCK_ELEMS;
    for (int kb = 0; kb < nkb; ++kb, blk += BLOCK_ELEMS) {
        uint4 x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) x[i] = *reinterpret_cast<const uint4*>(blk + poff[i]);
        float qv[NB][8];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const float* qp = qf + (int64_t)(b < B ? b : 0) * dpad + kb * KB + c * 8;
            float4 q0 = *reinterpret_cast<const float4*>(qp), q1 = *reinterpret_cast<const float4*>(qp + 4);
            qv[b][0] = q0.x; qv[b][1] = q0.y; qv[b][2] = q0.z; qv[b][3] = q0.w;
            qv[b][4] = q1.x; qv[b][5] = q1.y; qv[b][6] = q1.z; qv[b][7] = q1.w;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint32_t w[4] = {x[i].x, x[i].y, x[i].z, x[i].w};
            float e[8];
#pragma unroll
            for (int j = 0; j < 4; ++j) { e[2 * j] = ST::dec((uint16_t)(w[j] & 0xffff)); e[2 * j + 1] = ST::dec((uint16_t)(w[j] >> 16)); }
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[i][b] = fmaf(e[j], qv[b][j], acc[i][b]);
        }
    }
    // combine the 8 lanes of each row; afterwards lane c takes care of row group i == c
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = acc[i][b];
            v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64);
            acc[i][b] = v;
        }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (c != i) continue;
        int64_t id = t * TILE_ROWS + i * 32 + rbase;
        if (id >= N) continue;
        float inve = invnorm[id];
        const uint32_t tag = mask.tags ? mask.tags[id] : 0u;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b >= B) break;
            float v = acc[i][b] * inve;
            const bool ok = !mask.tags || eligible(tag, mask.allow[b], mask.exclude[b]);
            if (L.rho == 0)      // sparsest pass keeps every row at its own position, no counter (0 = empty slot)
                surv[(int64_t)b * SURV_CAP + (int64_t)blockIdx.x * TILE_ROWS + (id - t * TILE_ROWS)] = ok ? pack_key(v * invq[b], (int32_t)id) : 0ull;
            else if (ok && v >= thr[b]) append_survivor(v, invq[b], (int32_t)id, cnt + b, surv + (int64_t)b * SURV_CAP);
        }
    }
}

// fp32 stores: CH = 16 chunks of 4 elements per 256-byte segment.
template <int NB>
__global__ __launch_bounds__(256) void k_scan_gemv32(const float* __restrict__ store,
                                                     const float* __restrict__ invnorm,
                                                     const float* __restrict__ qf, const float* __restrict__ invq,
                                                     const float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                     uint64_t* __restrict__ surv, int64_t N, int nkb, int B,
                                                     Level L, Mask mask) {
    const int tid = threadIdx.x, c = tid & 15, rbase = tid >> 4;   // rbase 0..15
    const int64_t t = level_tile(L, blockIdx.x);
    const int dpad = nkb * KB;
    float acc[16][NB];
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[i][b] = 0.f;
    const float* blk = store + t * nkb * (int64_t)BLOCK_ELEMS + rbase * KB + c * 4;
    for (int kb = 0; kb < nkb; ++kb, blk += BLOCK_ELEMS) {
        float4 x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = *reinterpret_cast<const float4*>(blk + i * 16 * KB);
        float4 qv[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b)
            qv[b] = *reinterpret_cast<const float4*>(qf + (int64_t)(b < B ? b : 0) * dpad + kb * KB + c * 4);
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float a = acc[i][b];
                a = fmaf(x[i].x, qv[b].x, a); a = fmaf(x[i].y, qv[b].y, a);
                a = fmaf(x[i].z, qv[b].z, a); a = fmaf(x[i].w, qv[b].w, a);
                acc[i][b] = a;
            }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i)
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            float v = acc[i][b];
            v += __shfl_xor(v, 1, 64); v += __shfl_xor(v, 2, 64); v += __shfl_xor(v, 4, 64); v += __shfl_xor(v, 8, 64);
            acc[i][b] = v;
        }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (c != i) continue;
        int64_t id = t * TILE_ROWS + i * 16 + rbase;
        if (id >= N) continue;
        float inve = invnorm[id];
        const uint32_t tag = mask.tags ? mask.tags[id] : 0u;
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            if (b >= B) break;
            float v = acc[i][b] * inve;
            const bool ok = !mask.tags || eligible(tag, mask.allow[b], mask.exclude[b]);
            if (L.rho == 0)      // sparsest pass keeps every row at its own position, no counter (0 = empty slot)
                surv[(int64_t)b * SURV_CAP + (int64_t)blockIdx.x * TILE_ROWS + (id - t * TILE_ROWS)] = ok ? pack_key(v * invq[b], (int32_t)id) : 0ull;
            else if (ok && v >= thr[b]) append_survivor(v, invq[b], (int32_t)id, cnt + b, surv + (int64_t)b * SURV_CAP);
        }
    }
}

}  // namespace evk
