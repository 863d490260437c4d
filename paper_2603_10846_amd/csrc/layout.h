// Embedding-store layout in HBM and small device helpers shared by the kernels.
//
// The bank (Sec. 3.1 of the paper: a memory that only grows) is scanned front to back by every
// retrieval (Sec. 3.2, dense recall), so its layout is chosen for that scan, not for row access:
//
//   store = [tile t = id / 256][k-block kb = k / 64][row r = id % 256][64 elements]
//
// One (t, kb) block is a contiguous 32 KB (16-bit elements) or 64 KB (fp32) piece that a workgroup
// streams with 16-byte loads per lane, fully coalesced, and that can be copied into LDS verbatim.
// For 16-bit elements the eight 16-byte chunks of a row's 128-byte segment are XOR-swizzled by the
// row index, so that the LDS image serves MFMA operand reads (32 rows x one chunk per half-wave)
// without bank conflicts and needs no address arithmetic when it is staged.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace evk {

constexpr int TILE_ROWS = 256;            // bank rows per tile
constexpr int KB = 64;                    // elements per k-block
constexpr int BLOCK_ELEMS = TILE_ROWS * KB;
constexpr int SURV_CAP = 8192;            // survivor slots per query
constexpr int KEEP_MAX = 512;             // padded size of the selected list (k1 + guard band) for pools up to 256
constexpr int BIG_K1_MAX = 2048;          // largest pool
constexpr int SMALL_K1_MAX = 256;         // largest pool of the one-entry-per-lane value filter (k_rerank)
// room for the selected list of a pool of k1: the pool plus a guard band of near-ties
__host__ __device__ constexpr int keep_of(int k1) { return k1 <= 256 ? KEEP_MAX : k1 + 256; }

// physical 16-byte chunk index of logical chunk c (0..7) in row r (16-bit stores only)
__host__ __device__ __forceinline__ int swz16(int c, int r) { return c ^ ((r >> 1) & 7); }

// element offset of logical 8-element chunk c8 (k = 8*c8 ..) of entry id, 16-bit store
__host__ __device__ __forceinline__ int64_t off16(int64_t id, int c8, int nkb) {
    int64_t t = id >> 8; int r = (int)(id & 255); int kb = c8 >> 3; int c = c8 & 7;
    return (t * nkb + kb) * (int64_t)BLOCK_ELEMS + r * KB + swz16(c, r) * 8;
}
// element offset of logical 4-element chunk c4 (k = 4*c4 ..) of entry id, fp32 store
__host__ __device__ __forceinline__ int64_t off32(int64_t id, int c4, int nkb) {
    int64_t t = id >> 8; int r = (int)(id & 255); int kb = c4 >> 4; int c = c4 & 15;
    return (t * nkb + kb) * (int64_t)BLOCK_ELEMS + r * KB + c * 4;
}

// Bank rows are read once per retrieve and written once per append, in streams far larger than the
// caches: such accesses carry the non-temporal hint, so that they do not displace what is re-used
// (queries, thresholds, lists).  Measured on MI355X: a read-only pass over a 2 GB store 6.05 -> 6.89
// TB/s, the 64K x 4096 append 5.45 -> 6.2 TB/s, the densest scan pass at one query 0.338 -> 0.293 ms.
typedef __attribute__((ext_vector_type(4))) uint32_t stream_u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t stream_u32x2;
typedef __attribute__((ext_vector_type(4))) float stream_f32x4;
__device__ __forceinline__ stream_u32x4 stream_load16(const void* p) {
    return __builtin_nontemporal_load(static_cast<const stream_u32x4*>(p));
}
__device__ __forceinline__ float4 stream_load_float4(const float* p) {
    const stream_f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const stream_f32x4*>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ void stream_store8(void* p, uint32_t lo, uint32_t hi) {
    const stream_u32x2 t = {lo, hi};
    __builtin_nontemporal_store(t, static_cast<stream_u32x2*>(p));
}
__device__ __forceinline__ void stream_store_float4(float* p, float4 v) {
    const stream_f32x4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<stream_f32x4*>(p));
}

// ---- order-preserving packing of (similarity, id): larger key = better; lower id wins ties ----
__device__ __forceinline__ uint32_t f2ord(float f) {
    uint32_t u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord2f(uint32_t o) {
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}
__device__ __forceinline__ uint64_t pack_key(float sim, int32_t id) {
    return ((uint64_t)f2ord(sim) << 32) | (uint64_t)(0xffffffffu - (uint32_t)id);
}
__device__ __forceinline__ int32_t key_id(uint64_t k) { return (int32_t)(0xffffffffu - (uint32_t)k); }
__device__ __forceinline__ float key_sim(uint64_t k) { return ord2f((uint32_t)(k >> 32)); }

// ---- element conversion, round-to-nearest-even ----
__device__ __forceinline__ uint16_t f2bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
__device__ __forceinline__ uint16_t f2f16_rne(float x) {
    _Float16 h = (_Float16)x;              // v_cvt_f16_f32, round-to-nearest-even
    return *reinterpret_cast<uint16_t*>(&h);
}
__device__ __forceinline__ float f16_to_f(uint16_t h) {
    _Float16 v = *reinterpret_cast<_Float16*>(&h);
    return (float)v;
}

struct BF16 { static constexpr int id = 1;
    static __device__ __forceinline__ uint16_t enc(float x) { return f2bf16_rne(x); }
    static __device__ __forceinline__ float dec(uint16_t h) { return bf16_to_f(h); } };
struct F16 { static constexpr int id = 2;
    static __device__ __forceinline__ uint16_t enc(float x) { return f2f16_rne(x); }
    static __device__ __forceinline__ float dec(uint16_t h) { return f16_to_f(h); } };

// Which tiles a scan level covers.  The bank is scanned in a few passes of increasing density;
// each pass only has to beat the k1-th best similarity found by the sparser passes before it.
// Level tiles: t = u * stride with u in [0, U); for every level but the sparsest, the u that are
// multiples of rho (they belong to a sparser level) are left out.
struct Level {
    int stride;     // tile stride S of this level
    int rho;        // parent stride / S  (0 for the sparsest level)
    int ntiles;     // tiles this level scans
};
// Typed / masked retrieval (Sec. 3.2: the bank holds items of several types; Sec. 4.3: entries that
// stem from held-out operators are excluded).  Every entry carries a 32-bit tag: type = tag & 0xff
// (types 0..31), group = tag >> 8.  A query names the types it accepts as a bit mask and at most one
// group to leave out (0xffffffff: none).  tags == nullptr means no filtering.
struct Mask {
    const uint32_t* tags;      // [capacity]
    const uint32_t* allow;     // [B] bit t set = type t accepted
    const uint32_t* exclude;   // [B] group to leave out
};
__host__ __device__ __forceinline__ bool eligible(uint32_t tag, uint32_t allow, uint32_t exclude) {
    return ((allow >> (tag & 31u)) & 1u) != 0 && (tag & 0xe0u) == 0 && (tag >> 8) != exclude;
}

__host__ __device__ __forceinline__ int64_t level_tile(const Level& L, int j) {
    int64_t u = L.rho ? ((int64_t)(j / (L.rho - 1)) * L.rho + (j % (L.rho - 1)) + 1) : j;
    return u * L.stride;
}

}  // namespace evk
