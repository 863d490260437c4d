// Ingest kernels: append rows to the tiled store, read them back, prepare a batch of queries.
#pragma once
#include "layout.h"

namespace evk {

__device__ __forceinline__ float wave_sum_f(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// Memory growth rule of Sec. 3.1: entry first_id + row gets embedding emb[row], rounded to the
// store's element type; the inverse L2 norm of the *stored* values is kept beside it (fp32, used
// only by the scan's filter; the value filter recomputes norms in fp64) and both Q tables get their
// initial value.  One wavefront per row.  A lane takes 4 consecutive elements per step: its 16-byte
// load is one contiguous 1 KB read per wavefront, its 8-byte store half of a 16-byte chunk of the
// tiled store (two neighbouring lanes fill a chunk), four steps in flight at a time.  Both are streamed
// (non-temporal, see layout.h).
template <typename ST>  // BF16, F16 (uint16_t storage) ; fp32 handled by the overload below
__global__ __launch_bounds__(256) void k_append16(const float* __restrict__ emb, int64_t n, int d, int nkb,
                                                  int64_t first_id, uint16_t* __restrict__ store,
                                                  float* __restrict__ invnorm, float* __restrict__ qtab,
                                                  int64_t capacity, const float* __restrict__ q0d,
                                                  const float* __restrict__ q0r) {
    int lane = threadIdx.x & 63;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    int64_t id = first_id + row;
    const float* src = emb + row * (int64_t)d;
    float ssq = 0.f;
    const int ngroups = nkb * 16;                       // groups of 4 elements, padding included
    for (int g0 = lane; g0 < ngroups; g0 += 4 * 64) {
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = g0 + 64 * u;
            v[u] = (g < ngroups && g * 4 < d) ? stream_load_float4(src + g * 4) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int g = g0 + 64 * u;
            if (g >= ngroups) break;
            const uint16_t h0 = ST::enc(v[u].x), h1 = ST::enc(v[u].y), h2 = ST::enc(v[u].z), h3 = ST::enc(v[u].w);
            const float w0 = ST::dec(h0), w1 = ST::dec(h1), w2 = ST::dec(h2), w3 = ST::dec(h3);
            ssq += w0 * w0; ssq += w1 * w1; ssq += w2 * w2; ssq += w3 * w3;
            uint2 pk;
            pk.x = h0 | ((uint32_t)h1 << 16); pk.y = h2 | ((uint32_t)h3 << 16);
            stream_store8(store + off16(id, g >> 1, nkb) + (g & 1) * 4, pk.x, pk.y);
        }
    }
    ssq = wave_sum_f(ssq);
    if (lane == 0) {
        invnorm[id] = (float)(1.0 / sqrt((double)ssq));
        qtab[id] = q0d ? q0d[row] : 0.f;
        qtab[capacity + id] = q0r ? q0r[row] : 0.f;
    }
}

__global__ __launch_bounds__(256) void k_append32(const float* __restrict__ emb, int64_t n, int d, int nkb,
                                                  int64_t first_id, float* __restrict__ store,
                                                  float* __restrict__ invnorm, float* __restrict__ qtab,
                                                  int64_t capacity, const float* __restrict__ q0d,
                                                  const float* __restrict__ q0r) {
    int lane = threadIdx.x & 63;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    int64_t id = first_id + row;
    const float* src = emb + row * (int64_t)d;
    float ssq = 0.f;
    for (int c4 = lane; c4 < nkb * 16; c4 += 64) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 * 4 < d) a = stream_load_float4(src + c4 * 4);
        ssq += a.x * a.x + a.y * a.y + a.z * a.z + a.w * a.w;
        stream_store_float4(store + off32(id, c4, nkb), a);
    }
    ssq = wave_sum_f(ssq);
    if (lane == 0) {
        invnorm[id] = (float)(1.0 / sqrt((double)ssq));
        qtab[id] = q0d ? q0d[row] : 0.f;
        qtab[capacity + id] = q0r ? q0r[row] : 0.f;
    }
}

// Stored rows first .. first+n widened to fp32, row-major [n][d].
template <typename ST>
__global__ __launch_bounds__(256) void k_read_rows16(const uint16_t* __restrict__ store, int64_t first, int64_t n,
                                                     int d, int nkb, float* __restrict__ dst) {
    int lane = threadIdx.x & 63;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    for (int c8 = lane; c8 * 8 < d; c8 += 64) {
        uint4 pk = *reinterpret_cast<const uint4*>(store + off16(first + row, c8, nkb));
        uint32_t w[4] = {pk.x, pk.y, pk.z, pk.w};
        float* o = dst + row * (int64_t)d + c8 * 8;
#pragma unroll
        for (int i = 0; i < 4; ++i) { o[2 * i] = ST::dec((uint16_t)(w[i] & 0xffff)); o[2 * i + 1] = ST::dec((uint16_t)(w[i] >> 16)); }
    }
}
__global__ __launch_bounds__(256) void k_read_rows32(const float* __restrict__ store, int64_t first, int64_t n,
                                                     int d, int nkb, float* __restrict__ dst) {
    int lane = threadIdx.x & 63;
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= n) return;
    for (int c4 = lane; c4 * 4 < d; c4 += 64)
        *reinterpret_cast<float4*>(dst + row * (int64_t)d + c4 * 4) =
            *reinterpret_cast<const float4*>(store + off32(first + row, c4, nkb));
}

// Read-only pass over the stored rows, nothing else: every 16-byte piece of the store is loaded once and
// folded into a checksum.  It measures what a scan of this bank can reach at best on the machine at
// hand (the similarity scan of Sec. 3.2 has to read the same bytes once per retrieve).
// Access pattern of the scan itself: a workgroup takes whole contiguous 64 KB pieces, round-robin, each
// lane 16 independent 16-byte loads (one load instruction of the workgroup covers 4 KB).
__global__ __launch_bounds__(256) void k_read_probe(const uint4* __restrict__ p, int64_t n16, uint32_t* __restrict__ checksum) {
    constexpr int PIECE = 4096;                          // 16-byte units per 64 KB piece
    const int64_t pieces = n16 / PIECE;
    uint32_t acc = 0;
    for (int64_t c = blockIdx.x; c < pieces; c += gridDim.x) {
        const uint4* q = p + c * PIECE + threadIdx.x;
        uint4 v[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) { const stream_u32x4 t = stream_load16(q + u * 256); v[u] = make_uint4(t.x, t.y, t.z, t.w); }
#pragma unroll
        for (int u = 0; u < 16; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    for (int64_t i = pieces * PIECE + (int64_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (int64_t)gridDim.x * 256) {
        const uint4 v = p[i];
        acc ^= v.x ^ v.y ^ v.z ^ v.w;
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc ^= __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) atomicXor(checksum, acc);
}

// Query preparation (Sec. 3.2, the query side of dense retrieval): round each query to the store's
// element type, keep it widened (fp32, row-major, zero-padded to the k-block multiple) for the
// GEMV scan and the fp64 re-score, and in the operand layout of the MFMA scan
//   qop = [kb][Bpad][64 elements], 16-byte chunks swizzled like the bank rows, plus one all-zero
//         k-block at kb = nkb                                                        (16-bit stores)
//   qop = [kb][half h][Bpad][32 hi | 32 lo bf16], same swizzle                      (fp32 stores:
//         the query is split as hi + lo in bf16 so that the scan can use bf16 MFMA)
// plus its inverse norm (fp32 and fp64).  Also resets the per-query threshold and presets the
// survivor count to the number of rows of the sparsest scan pass, which keeps every row.
// One workgroup per padded query slot; slots >= B become all-zero queries that never pass a filter.
template <int DT>
__global__ __launch_bounds__(256) void k_prep_queries(const float* __restrict__ q, int B, int Bpad, int d, int nkb,
                                                      float* __restrict__ qf, uint16_t* __restrict__ qop,
                                                      float* __restrict__ invq, double* __restrict__ invq64,
                                                      float* __restrict__ thr, uint32_t* __restrict__ cnt,
                                                      uint32_t* __restrict__ flags, uint32_t cnt0) {
    int b = blockIdx.x, tid = threadIdx.x;
    int dpad = nkb * KB;
    __shared__ double red[256];
    double ssq = 0.0;
    for (int c8 = tid; c8 < nkb * 8; c8 += 256) {
        float v[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = (b < B && c8 * 8 + i < d) ? q[(int64_t)b * d + c8 * 8 + i] : 0.f;
        int kb = c8 >> 3, c = c8 & 7;
        if (DT == 0) {
            // fp32 store: keep the value; operand = bf16 hi + bf16 lo
            uint16_t hi[8], lo[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                hi[i] = f2bf16_rne(v[i]);
                lo[i] = f2bf16_rne(v[i] - bf16_to_f(hi[i]));
                ssq += (double)v[i] * (double)v[i];
            }
            // half h = c / 4 of the k-block; inside it logical chunk (c % 4) is hi, 4 + (c % 4) is lo
            int h = c >> 2, cc = c & 3;
            uint16_t* base = qop + (((int64_t)kb * 2 + h) * Bpad + b) * KB;
            uint4 ph, pl;
            ph.x = hi[0] | ((uint32_t)hi[1] << 16); ph.y = hi[2] | ((uint32_t)hi[3] << 16);
            ph.z = hi[4] | ((uint32_t)hi[5] << 16); ph.w = hi[6] | ((uint32_t)hi[7] << 16);
            pl.x = lo[0] | ((uint32_t)lo[1] << 16); pl.y = lo[2] | ((uint32_t)lo[3] << 16);
            pl.z = lo[4] | ((uint32_t)lo[5] << 16); pl.w = lo[6] | ((uint32_t)lo[7] << 16);
            *reinterpret_cast<uint4*>(base + swz16(cc, b & 255) * 8) = ph;
            *reinterpret_cast<uint4*>(base + swz16(4 + cc, b & 255) * 8) = pl;
        } else {
            uint16_t h[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                h[i] = DT == 1 ? f2bf16_rne(v[i]) : f2f16_rne(v[i]);
                v[i] = DT == 1 ? bf16_to_f(h[i]) : f16_to_f(h[i]);
                ssq += (double)v[i] * (double)v[i];
            }
            uint4 pk;
            pk.x = h[0] | ((uint32_t)h[1] << 16); pk.y = h[2] | ((uint32_t)h[3] << 16);
            pk.z = h[4] | ((uint32_t)h[5] << 16); pk.w = h[6] | ((uint32_t)h[7] << 16);
            *reinterpret_cast<uint4*>(qop + ((int64_t)kb * Bpad + b) * KB + swz16(c, b & 255) * 8) = pk;
        }
        float* o = qf + (int64_t)b * dpad + c8 * 8;
        *reinterpret_cast<float4*>(o) = make_float4(v[0], v[1], v[2], v[3]);
        *reinterpret_cast<float4*>(o + 4) = make_float4(v[4], v[5], v[6], v[7]);
    }
    // one all-zero k-block behind the last one: the MFMA scan pairs it with a repeated bank block
    // when it pads an odd number of k-steps to an even one
    if (DT != 0 && tid < 8) *reinterpret_cast<uint4*>(qop + ((int64_t)nkb * Bpad + b) * KB + tid * 8) = make_uint4(0, 0, 0, 0);
    red[tid] = ssq;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
    if (tid == 0) {
        bool live = b < B;
        double inv = live ? 1.0 / sqrt(red[0]) : 0.0;
        invq64[b] = inv;
        invq[b] = (float)inv;
        // "No threshold yet" is a finite floor below every reachable value (the scan compares
        // dot * invnorm, which lies in [-|q|, |q|]); empty slots get a threshold their all-zero query
        // can never reach.  Finite values keep the scan's arithmetic free of inf - inf.
        thr[b] = live ? (float)(-2.0 / inv) : 1.0f;
        cnt[b] = live ? cnt0 : 0u;     // rows the sparsest pass will write without counting
        flags[b] = 0u;                 // per-query status of this retrieve (bit 0: a survivor list overflowed)
    }
}

}  // namespace evk
