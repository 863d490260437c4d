// Host side of the evomem C ABI (include/evomem.h): argument checks, workspace carving, the scan
// plan, kernel dispatch.  Every step of the method runs in the kernels included below.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/evomem.h"
#include "k_ingest.h"
#include "k_scan_gemv.h"
#include "k_scan_mfma.h"
#include "k_select.h"
#include "k_rerank_big.h"
#include "k_reward.h"
#include "k_startpoint.h"
#include "k_update.h"
#include "layout.h"

using namespace evk;

static_assert(MEM_MAX_K1 == evk::BIG_K1_MAX, "header and kernels disagree on the largest pool");

namespace {

constexpr int MAX_PROFILE = 4096;
constexpr int GEMV_MAX_B = 4;       // fp32 stores: at most this many queries use the VALU scan

constexpr int MAX_DEVICES = 16;     // per-device set-up flags and scratch addresses are kept in arrays of this size

constexpr int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// Calls f with the store type as a compile-time constant (0 fp32, 1 bf16, 2 fp16: the kernels' DT).
template <class F>
void with_store_type(int dtype, F&& f) {
    if (dtype == MEM_F32) f(std::integral_constant<int, 0>{});
    else if (dtype == MEM_BF16) f(std::integral_constant<int, 1>{});
    else f(std::integral_constant<int, 2>{});
}

struct Workspace {   // byte offsets into a scratch area (the caller's workspace, or the library's own array)
    size_t counters, qf, qop, invq, invq64, thr, cnt, flags, surv, exact, total;
};

// A retrieve pads its batch to a multiple of its query tile (32 .. 256 queries), so the per-query
// arrays are sized for max_B rounded up to `bpad` (256 covers every tile).
constexpr Workspace carve(int d, int dtype, int max_B, int max_k1, int bpad = 256) {
    const int64_t dpad = round_up(d, KB), Bp = round_up(max_B, bpad);
    const size_t sizes[10] = {256, (size_t)Bp * dpad * 4,
                              (size_t)Bp * (dpad + KB) * (dtype == MEM_F32 ? 4 : 2),   // + one all-zero k-block
                              (size_t)Bp * 4, (size_t)Bp * 8, (size_t)Bp * 4, (size_t)Bp * 4, (size_t)Bp * 4,
                              (size_t)Bp * SURV_CAP * 8, (size_t)Bp * keep_of(max_k1) * 8};
    size_t at[11] = {};
    for (int i = 0; i < 10; ++i) at[i + 1] = (size_t)round_up((int64_t)(at[i] + sizes[i]), 256);
    return Workspace{at[0], at[1], at[2], at[3], at[4], at[5], at[6], at[7], at[8], at[9], at[10]};
}

// Where a retrieve keeps its intermediate results.
struct Scratch {
    unsigned char* base;
    Workspace w;
    int exact_stride;      // fp64 similarities per query
};

// Limits of mem_retrieve_static and the library's own scratch array for it (see the header).
constexpr int STATIC_MAX_B = 64, STATIC_MAX_K1 = 256, STATIC_MAX_D = 2048;
constexpr Workspace STATIC_W = carve(STATIC_MAX_D, MEM_F32, STATIC_MAX_B, STATIC_MAX_K1, STATIC_MAX_B);
constexpr size_t STATIC_SCRATCH_BYTES = STATIC_W.total;
static_assert(STATIC_SCRATCH_BYTES <= (6u << 20), "the built-in scratch array is meant to stay small");

bool shape_ok(int d, int dtype, int64_t capacity) {
    return d >= 8 && d <= 16384 && d % 8 == 0 && dtype >= MEM_F32 && dtype <= MEM_F16 && capacity >= 1 &&
           capacity <= 2147483647ll - 256;
}


}  // namespace

struct evomem {
    int d, dtype, nkb, device, max_B, max_k1;
    int64_t capacity, N;
    void* store;
    float* invnorm;
    float* q;
    unsigned char* ws;
    Workspace w;
    bool lds_attr_set;
    // profiling
    bool prof_on;
    int prof_n;
    uint32_t* tags = nullptr;   // per-entry tags of typed / masked retrieval (caller's buffer), or null
    const uint32_t* last_flags = nullptr;   // per-query status words of the latest retrieve (in the scratch it used)
    int last_B = 0;
    std::vector<hipEvent_t> ev;
    std::vector<int64_t> prof_rows;
};

// Clears a few words on the stream (a kernel, not a memset: callers may record their calls into a HIP graph).
__global__ void k_clear_words(uint32_t* p, int n) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) p[i] = 0u;
}

#define HIPCHK(x) do { if ((x) != hipSuccess) return MEM_EHIP; } while (0)
#define LAUNCHCHK() do { if (hipGetLastError() != hipSuccess) return MEM_EHIP; } while (0)

extern "C" {

size_t mem_store_bytes(int d, int dtype, int64_t capacity) {
    if (!shape_ok(d, dtype, capacity)) return 0;
    return (size_t)round_up(capacity, TILE_ROWS) * (size_t)round_up(d, KB) * (dtype == MEM_F32 ? 4 : 2);
}

size_t mem_workspace_bytes(int d, int dtype, int64_t capacity, int max_B, int max_k1) {
    if (!shape_ok(d, dtype, capacity) || max_B < 1 || max_B > MEM_MAX_B || max_k1 < 1 || max_k1 > MEM_MAX_K1) return 0;
    return carve(d, dtype, max_B, max_k1).total;
}

int mem_create(evomem_t** out, int d, int dtype, int64_t capacity, void* store_dev, float* invnorm_dev,
               float* q_dev, void* workspace_dev, size_t workspace_bytes, int max_B, int max_k1, int device) {
    if (!out) return MEM_EINVAL;
    *out = nullptr;
    if (!shape_ok(d, dtype, capacity) || !store_dev || !invnorm_dev || !q_dev || !workspace_dev) return MEM_EINVAL;
    if (max_B < 1 || max_B > MEM_MAX_B || max_k1 < 1 || max_k1 > MEM_MAX_K1 || device < 0 || device >= MAX_DEVICES) return MEM_EINVAL;
    if (((uintptr_t)store_dev | (uintptr_t)workspace_dev) & 255) return MEM_EINVAL;
    Workspace w = carve(d, dtype, max_B, max_k1);
    if (workspace_bytes < w.total) return MEM_EWORKSPACE;
    evomem* h = new (std::nothrow) evomem();
    if (!h) return MEM_EHIP;
    h->d = d; h->dtype = dtype; h->nkb = (int)(round_up(d, KB) / KB); h->device = device;
    h->max_B = max_B; h->max_k1 = max_k1; h->capacity = capacity; h->N = 0;
    h->store = store_dev; h->invnorm = invnorm_dev; h->q = q_dev;
    h->ws = static_cast<unsigned char*>(workspace_dev); h->w = w;
    h->lds_attr_set = false; h->prof_on = false; h->prof_n = 0;
    if (hipSetDevice(device) != hipSuccess || hipMemsetAsync(h->ws + w.counters, 0, 256, nullptr) != hipSuccess ||
        hipStreamSynchronize(nullptr) != hipSuccess) {
        delete h;
        return MEM_EHIP;
    }
    *out = h;
    return MEM_OK;
}

int mem_destroy(evomem_t* h) {
    if (!h) return MEM_EINVAL;
    for (hipEvent_t e : h->ev) (void)hipEventDestroy(e);
    delete h;
    return MEM_OK;
}

int mem_size(const evomem_t* h, int64_t* n_out) {
    if (!h || !n_out) return MEM_EINVAL;
    *n_out = h->N;
    return MEM_OK;
}

int mem_append(evomem_t* h, const float* emb_dev, int64_t n, const float* q0d, const float* q0r,
               int64_t* first_id_out, void* hip_stream) {
    if (!h || n < 0 || (n > 0 && !emb_dev)) return MEM_EINVAL;
    if (h->N + n > h->capacity) return MEM_ECAPACITY;
    if (first_id_out) *first_id_out = h->N;
    if (n == 0) return MEM_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    dim3 grid((unsigned)((n + 3) / 4)), block(256);
    if (h->dtype == MEM_F32)
        hipLaunchKernelGGL(k_append32, grid, block, 0, st, emb_dev, n, h->d, h->nkb, h->N, (float*)h->store,
                           h->invnorm, h->q, h->capacity, q0d, q0r);
    else if (h->dtype == MEM_BF16)
        hipLaunchKernelGGL(k_append16<BF16>, grid, block, 0, st, emb_dev, n, h->d, h->nkb, h->N, (uint16_t*)h->store,
                           h->invnorm, h->q, h->capacity, q0d, q0r);
    else
        hipLaunchKernelGGL(k_append16<F16>, grid, block, 0, st, emb_dev, n, h->d, h->nkb, h->N, (uint16_t*)h->store,
                           h->invnorm, h->q, h->capacity, q0d, q0r);
    LAUNCHCHK();
    h->N += n;
    return MEM_OK;
}

int mem_read_q(evomem_t* h, int stage, int64_t first, int64_t n, float* dst_dev, void* hip_stream) {
    if (!h || (stage != 0 && stage != 1) || first < 0 || n < 0 || first + n > h->N || (n > 0 && !dst_dev)) return MEM_EINVAL;
    if (n == 0) return MEM_OK;
    HIPCHK(hipMemcpyAsync(dst_dev, h->q + stage * h->capacity + first, (size_t)n * 4, hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(hip_stream)));
    return MEM_OK;
}

int mem_read_rows(evomem_t* h, int64_t first, int64_t n, float* dst_dev, void* hip_stream) {
    if (!h || first < 0 || n < 0 || first + n > h->N || (n > 0 && !dst_dev)) return MEM_EINVAL;
    if (n == 0) return MEM_OK;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    dim3 grid((unsigned)((n + 3) / 4)), block(256);
    if (h->dtype == MEM_F32)
        hipLaunchKernelGGL(k_read_rows32, grid, block, 0, st, (const float*)h->store, first, n, h->d, h->nkb, dst_dev);
    else if (h->dtype == MEM_BF16)
        hipLaunchKernelGGL(k_read_rows16<BF16>, grid, block, 0, st, (const uint16_t*)h->store, first, n, h->d, h->nkb, dst_dev);
    else
        hipLaunchKernelGGL(k_read_rows16<F16>, grid, block, 0, st, (const uint16_t*)h->store, first, n, h->d, h->nkb, dst_dev);
    LAUNCHCHK();
    return MEM_OK;
}

int mem_counters(evomem_t* h, int64_t* skipped_ids, int64_t* overflows) {
    if (!h) return MEM_EINVAL;
    uint32_t c[2] = {0, 0};
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMemcpy(c, h->ws + h->w.counters, 8, hipMemcpyDeviceToHost));
    if (skipped_ids) *skipped_ids = c[0];
    if (overflows) *overflows = c[1];
    return MEM_OK;
}

int mem_read_probe(evomem_t* h, uint32_t* checksum_dev, int64_t* bytes_out, void* hip_stream) {
    if (!h || !checksum_dev) return MEM_EINVAL;
    const int64_t bytes = round_up(h->N, TILE_ROWS) * (int64_t)h->nkb * KB * (h->dtype == MEM_F32 ? 4 : 2);
    if (bytes_out) *bytes_out = bytes;
    if (bytes == 0) return MEM_OK;
    int cus = 0;
    HIPCHK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device));
    // two workgroups per compute unit: measured 6.2 TB/s on a 24 GB store, against 5.7-5.8 TB/s with four or eight
    hipLaunchKernelGGL(k_read_probe, dim3((unsigned)(cus * 2)), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       (const uint4*)h->store, bytes / 16, checksum_dev);
    LAUNCHCHK();
    return MEM_OK;
}

int mem_profile_enable(evomem_t* h, int on) {
    if (!h) return MEM_EINVAL;
    if (on && h->ev.empty()) {
        h->ev.resize(2 * MAX_PROFILE);
        h->prof_rows.resize(MAX_PROFILE);
        for (size_t i = 0; i < h->ev.size(); ++i)
            if (hipEventCreate(&h->ev[i]) != hipSuccess) {       // leave no half-built set behind
                for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(h->ev[j]);
                h->ev.clear();
                h->prof_rows.clear();
                return MEM_EHIP;
            }
    }
    h->prof_on = on != 0;      // the records kept so far stay until they are read
    return MEM_OK;
}

int mem_profile_read(evomem_t* h, int capacity, int* n_out, float* ms_out, int64_t* rows_out) {
    if (!h || capacity < 0 || !n_out || (capacity > 0 && (!ms_out || !rows_out))) return MEM_EINVAL;
    HIPCHK(hipDeviceSynchronize());
    int n = h->prof_n < capacity ? h->prof_n : capacity;
    for (int i = 0; i < n; ++i) {
        HIPCHK(hipEventElapsedTime(&ms_out[i], h->ev[2 * i], h->ev[2 * i + 1]));
        rows_out[i] = h->prof_rows[i];
    }
    *n_out = n;
    h->prof_n = 0;
    return MEM_OK;
}

// the normaliser's statistics live in the zero-initialised counter block: double[2 stages][3] at byte 64
static double* reward_state(evomem_t* h, int stage) { return reinterpret_cast<double*>(h->ws + h->w.counters + 64) + 3 * stage; }

int mem_shape_rewards(evomem_t* h, int stage, const unsigned char* feasible_dev, const float* latency_dev,
                      const float* best_latency_dev, int64_t M, int normalise, float sigma_min, float clip,
                      float* rewards_out_dev, void* hip_stream) {
    if (!h || (stage != 0 && stage != 1) || M < 0 || (normalise && !(sigma_min > 0.f)) || !(clip >= 0.f)) return MEM_EINVAL;
    if (M == 0) return MEM_OK;
    if (!feasible_dev || !rewards_out_dev || (stage == 1 && (!latency_dev || !best_latency_dev))) return MEM_EINVAL;
    hipLaunchKernelGGL(k_shape_rewards, dim3(1), dim3(1024), 0, static_cast<hipStream_t>(hip_stream), stage, feasible_dev,
                       latency_dev, best_latency_dev, M, normalise, (double)sigma_min, (double)clip, reward_state(h, stage),
                       rewards_out_dev);
    LAUNCHCHK();
    return MEM_OK;
}

int mem_reward_stats(evomem_t* h, int stage, double* count, double* mean, double* sigma) {
    if (!h || (stage != 0 && stage != 1) || !count || !mean || !sigma) return MEM_EINVAL;
    double st[3];
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMemcpy(st, reward_state(h, stage), sizeof(st), hipMemcpyDeviceToHost));
    *count = st[0];
    *mean = st[0] > 0 ? st[1] / st[0] : 0.0;
    const double var = st[0] > 0 ? st[2] / st[0] - (*mean) * (*mean) : 0.0;
    *sigma = var > 0 ? sqrt(var) : 0.0;
    return MEM_OK;
}

int mem_reward_stats_reset(evomem_t* h, int stage, void* hip_stream) {
    if (!h || (stage != 0 && stage != 1)) return MEM_EINVAL;
    hipLaunchKernelGGL(k_clear_words, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream),
                       reinterpret_cast<uint32_t*>(reward_state(h, stage)), (int)(3 * sizeof(double) / sizeof(uint32_t)));
    LAUNCHCHK();
    return MEM_OK;
}

int mem_restore(evomem_t* h, int64_t n) {
    if (!h || n < 0) return MEM_EINVAL;
    if (n > h->capacity) return MEM_ECAPACITY;
    h->N = n;
    return MEM_OK;
}

const char* mem_strerror(int s) {
    switch (s) {
        case MEM_OK: return "ok";
        case MEM_EINVAL: return "invalid argument";
        case MEM_ECAPACITY: return "bank capacity exceeded";
        case MEM_EWORKSPACE: return "workspace too small";
        case MEM_EHIP: return "HIP runtime error";
        case MEM_ESTATE: return "handle in unusable state";
        default: return "unknown status";
    }
}

}  // extern "C"

namespace {

// Scan plan: tile strides of the passes, sparsest first.  The sparsest pass has no threshold, so it
// may cover at most SURV_CAP rows, and it is made as large as that allows (a larger sample gives the
// next pass a tighter threshold).  Each denser pass divides the stride by `ratio`, chosen so that
// about k1 * ratio rows (a quarter of the survivor slots) are expected to pass its threshold; the
// step up to the sparsest pass is whatever factor <= ratio fills its row budget.
// (at most 24 passes: every step divides the stride by at least 2 and a bank has fewer than 2^23 tiles;
// kept in a fixed array so that a retrieve allocates nothing on the host either)
constexpr int MAX_LEVELS = 24;
struct Plan { int n; Level lv[MAX_LEVELS]; };
Plan plan_levels(int64_t N, int k1) {
    const int nt = (int)((N + TILE_ROWS - 1) / TILE_ROWS);
    const int cap_tiles = SURV_CAP / TILE_ROWS;
    int ratio = SURV_CAP / (4 * k1);
    if (ratio > 16) ratio = 16;
    if (ratio < 2) ratio = 2;
    int strides[MAX_LEVELS] = {1}, ns = 1;
    for (;;) {
        const int U = (nt + strides[ns - 1] - 1) / strides[ns - 1];
        if (U <= cap_tiles) break;
        const int need = (U + cap_tiles - 1) / cap_tiles;          // >= 2
        strides[ns] = strides[ns - 1] * (need < ratio ? need : ratio);
        ++ns;
    }
    Plan p{};
    for (int i = ns - 1; i >= 0; --i) {
        Level L;
        L.stride = strides[i];
        const int U = (nt + L.stride - 1) / L.stride;
        if (i == ns - 1) { L.rho = 0; L.ntiles = U; }
        else { L.rho = strides[i + 1] / strides[i]; L.ntiles = U - (U + L.rho - 1) / L.rho; }
        if (L.ntiles > 0) p.lv[p.n++] = L;
    }
    return p;
}

template <int DT, int MQ, int WQ, int MR, int WR, bool MASKED, bool STREAM = true>
int launch_mfma(evomem* h, const Scratch& sc, hipStream_t st, int Bp, const Level& L, int k1, const Mask& mask, int B) {
    constexpr int QT = 32 * MQ * WQ;
    constexpr int lds = scan_mfma_lds_bytes<QT, MASKED>();
    auto kern = k_scan_mfma<DT, MQ, WQ, MR, WR, MASKED, STREAM>;
    static int resident[MAX_DEVICES] = {};          // workgroups of this kernel the whole device holds at once
    if (!resident[h->device]) {
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, lds));
        int per_cu = 0, cus = 0;
        HIPCHK(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void*>(kern), 64 * WQ * WR, lds));
        HIPCHK(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, h->device));
        if (per_cu < 1 || cus < 8) return MEM_EHIP;
        resident[h->device] = per_cu * cus;
    }
    // persistent launch: per XCD, `groups` tile walkers for each of the nqt query tiles
    const int nqt = Bp / QT;
    int groups = resident[h->device] / 8 / nqt;
    if (groups < 1) groups = 1;
    if (groups > (L.ntiles + 7) / 8) groups = (L.ntiles + 7) / 8;
    dim3 grid((unsigned)(8 * nqt * groups)), block(64 * WQ * WR);
    // A pass is expected to keep about k1 * rho rows per query; spread over its tiles that is the
    // number of survivors a workgroup stages per tile.  It writes its list out at evenly spaced tiles,
    // as seldom as keeps the expected fill under 55 % of the list (a surplus takes the direct path).
    const double per_tile = L.rho ? (double)k1 * L.rho * QT / L.ntiles : 1.0;
    const int tiles_per_wg = (int)((L.ntiles + 8 * groups - 1) / (8 * groups));
    int n_flush = (int)std::ceil(tiles_per_wg * (per_tile + 1.0) / (0.55 * SCAN_LIST_CAP));
    if (n_flush < 1) n_flush = 1;
    int flush_every = (tiles_per_wg + n_flush - 1) / n_flush;
    if (flush_every < 1) flush_every = 1;
    if (flush_every > 64) flush_every = 64;
    unsigned char* ws = sc.base;
    hipLaunchKernelGGL(kern, grid, block, lds, st, (const void*)h->store, (const float*)h->invnorm,
                       (const uint16_t*)(ws + sc.w.qop), (const float*)(ws + sc.w.invq), (const float*)(ws + sc.w.thr),
                       (uint32_t*)(ws + sc.w.cnt), (uint64_t*)(ws + sc.w.surv), h->N, h->nkb, Bp, L, flush_every, mask, B);
    LAUNCHCHK();
    return MEM_OK;
}

template <int DT, bool MASKED>
int launch_mfma_dt(evomem* h, const Scratch& sc, hipStream_t st, int Bp, int qt, const Level& L, int k1, const Mask& mask, int B) {
    switch (qt) {
        case 32: return launch_mfma<DT, 1, 1, 2, 4, MASKED>(h, sc, st, Bp, L, k1, mask, B);
        case 64:
            // fp32 stores: 8 wavefronts, so that one wavefront's hi/lo split (vector ALU) overlaps the
            // MFMAs of the other one on its SIMD (measured 0.054 -> 0.047 ms on the 65,536 x 1024 bank)
            if constexpr (DT == 0) return launch_mfma<DT, 1, 2, 2, 4, MASKED>(h, sc, st, Bp, L, k1, mask, B);
            else return launch_mfma<DT, 2, 1, 2, 4, MASKED>(h, sc, st, Bp, L, k1, mask, B);
        case 128: return launch_mfma<DT, 2, 2, 2, 4, MASKED>(h, sc, st, Bp, L, k1, mask, B);   // 8 wavefronts, 64 x 64 each
        default:                                                                               // 8 wavefronts, 128 x 64 each
            // several query tiles share every bank tile through L2: no streaming hint on the bank loads then
            return Bp > qt ? launch_mfma<DT, 4, 2, 2, 4, MASKED, false>(h, sc, st, Bp, L, k1, mask, B)
                           : launch_mfma<DT, 4, 2, 2, 4, MASKED, true>(h, sc, st, Bp, L, k1, mask, B);
    }
}
template <bool MASKED>
int launch_mfma_any(evomem* h, const Scratch& sc, hipStream_t st, int Bp, int qt, const Level& L, int k1, const Mask& mask, int B) {
    return h->dtype == MEM_F32 ? launch_mfma_dt<0, MASKED>(h, sc, st, Bp, qt, L, k1, mask, B)
         : h->dtype == MEM_BF16 ? launch_mfma_dt<1, MASKED>(h, sc, st, Bp, qt, L, k1, mask, B)
                                : launch_mfma_dt<2, MASKED>(h, sc, st, Bp, qt, L, k1, mask, B);
}

template <int NB>
int launch_gemv(evomem* h, const Scratch& sc, hipStream_t st, int B, const Level& L, const Mask& mask) {
    unsigned char* ws = sc.base;
    const bool split = L.ntiles < 1024;        // few tiles: four workgroups per tile
    dim3 grid((unsigned)(split ? 4 * L.ntiles : L.ntiles)), block(256);
    const float* invq = (const float*)(ws + sc.w.invq);
    const float* thr = (const float*)(ws + sc.w.thr);
    const float* qf = (const float*)(ws + sc.w.qf);
    uint32_t* cnt = (uint32_t*)(ws + sc.w.cnt);
    uint64_t* surv = (uint64_t*)(ws + sc.w.surv);
    if (split)
        hipLaunchKernelGGL((k_scan_gemv32<NB, 4>), grid, block, 0, st, (const float*)h->store, (const float*)h->invnorm, qf, invq,
                           thr, cnt, surv, h->N, h->nkb, B, L, mask);
    else
        hipLaunchKernelGGL((k_scan_gemv32<NB, 16>), grid, block, 0, st, (const float*)h->store, (const float*)h->invnorm, qf, invq,
                           thr, cnt, surv, h->N, h->nkb, B, L, mask);
    LAUNCHCHK();
    return MEM_OK;
}

}  // namespace

extern "C" int mem_plan_levels(int64_t N, int k1, int* stride, int* rho, int* ntiles, int max_levels) {
    if (N < 1 || N > 2147483647ll - 256 || k1 < 1 || k1 > MEM_MAX_K1 || !stride || !rho || !ntiles || max_levels < 1) return -1;
    const Plan p = plan_levels(N, k1);
    for (int i = 0; i < p.n && i < max_levels; ++i) { stride[i] = p.lv[i].stride; rho[i] = p.lv[i].rho; ntiles[i] = p.lv[i].ntiles; }
    return p.n;
}

static int retrieve_impl(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                         int32_t* out_ids_dev, float* out_scores_dev, int32_t* out_cand_ids_dev,
                         float* out_cand_sims_dev, void* hip_stream, const EpsGreedy& eg, const Mask& mask,
                         const Scratch& sc, int max_B, int max_k1, bool exhaustive = false) {
    if (!h || B < 0 || B > max_B || (stage != 0 && stage != 1) || k1 < 1 || k2 < 1 || k2 > k1 || k1 > max_k1)
        return MEM_EINVAL;
    if (!(lambda >= 0.f && lambda <= 1.f)) return MEM_EINVAL;
    if ((out_cand_ids_dev == nullptr) != (out_cand_sims_dev == nullptr)) return MEM_EINVAL;
    if (B == 0) return MEM_OK;
    if (!queries_dev || !out_ids_dev || !out_scores_dev) return MEM_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    unsigned char* ws = sc.base;
    const bool gemv = B <= GEMV_MAX_B && h->dtype == MEM_F32;
    // query tile of the MFMA scan and padded batch
    int qt = B <= 32 ? 32 : B <= 64 ? 64 : B <= 128 ? 128 : 256;
    const int Bp = gemv ? B : (int)round_up(B, qt);
    float* qf = (float*)(ws + sc.w.qf);
    uint16_t* qop = (uint16_t*)(ws + sc.w.qop);
    float* invq = (float*)(ws + sc.w.invq);
    double* invq64 = (double*)(ws + sc.w.invq64);
    float* thr = (float*)(ws + sc.w.thr);
    uint32_t* cnt = (uint32_t*)(ws + sc.w.cnt);
    uint32_t* flags = (uint32_t*)(ws + sc.w.flags);
    uint64_t* surv = (uint64_t*)(ws + sc.w.surv);
    double* exact = (double*)(ws + sc.w.exact);
    const int exact_stride = sc.exact_stride;
    h->last_flags = flags;
    h->last_B = B;
    uint32_t* counters = (uint32_t*)(ws + sc.w.counters);

    Plan plan{};
    uint32_t cnt0 = 0;      // valid rows of the sparsest pass (a prefix of its last tile may be all that exists)
    if (h->N > 0 && !exhaustive) {
        plan = plan_levels(h->N, k1);
        const Level& L0 = plan.lv[0];
        const int64_t last = level_tile(L0, L0.ntiles - 1) * TILE_ROWS;
        const int64_t in_last = h->N - last < TILE_ROWS ? h->N - last : TILE_ROWS;
        cnt0 = (uint32_t)((int64_t)(L0.ntiles - 1) * TILE_ROWS + in_last);
    }
    with_store_type(h->dtype, [&](auto dt) {
        hipLaunchKernelGGL(k_prep_queries<decltype(dt)::value>, dim3(Bp), dim3(256), 0, st, queries_dev, B, Bp, h->d, h->nkb, qf, qop,
                           invq, invq64, thr, cnt, flags, cnt0);
    });
    LAUNCHCHK();

    // rounding margin of the scan's fp32 similarities
    float eps = (float)(h->nkb * KB) * 5.97e-8f + 1e-6f;
    if (h->dtype == MEM_F32 && !gemv) eps += 2e-5f;      // bf16 hi/lo split of fp32 values
    if (!gemv) eps += 2e-5f;                             // threshold * norm carried as 16-bit hi/lo pairs
    const float margin = 2.f * eps;

    // Pools of up to 128 with one workgroup per query in the gather (more than 128 queries): the last
    // selection, the re-scoring and the value filter run as one launch (measured on the 1M x 1024 bank at
    // 256 queries: see the kernel).
    const bool fused_tail = h->N > 0 && k1 <= 128 && B > 128 && !exhaustive;
    if (h->N > 0 && exhaustive) {
        // every entry's similarity is accumulated in fp64; the bank is walked in ranges that fit a list
        const int keep = keep_of(k1);
        const int64_t range_rows = (int64_t)((SURV_CAP - keep) / TILE_ROWS) * TILE_ROWS;
        int parts = 1;
        while (parts < 64 && B * parts < 512) parts <<= 1;       // few queries: each query's range is shared by many workgroups
        for (int64_t first = 0; first < h->N; first += range_rows) {
            const int n_new = (int)(h->N - first < range_rows ? h->N - first : range_rows);
            hipLaunchKernelGGL(k_exact_fill, dim3(B), dim3(256), 0, st, surv, cnt, (int32_t)first, n_new);
            LAUNCHCHK();
            dim3 kgrid((unsigned)B, (unsigned)parts);
            with_store_type(h->dtype, [&](auto dt) {
                hipLaunchKernelGGL(k_exact_keys<decltype(dt)::value>, kgrid, dim3(1024), 0, st, (const void*)h->store, (const float*)qf,
                                   (const double*)invq64, surv, (const uint32_t*)cnt, h->nkb, n_new);
            });
            LAUNCHCHK();
            hipLaunchKernelGGL(k_exact_select, dim3(B), dim3(1024), 0, st, surv, cnt, thr, (const float*)invq, counters, flags, k1, keep);
            LAUNCHCHK();
        }
    }
    if (h->N > 0 && !exhaustive) {
        for (int li = 0; li < plan.n; ++li) {
            const Level& L = plan.lv[li];
            const bool prof = h->prof_on && h->prof_n < MAX_PROFILE;
            if (prof) HIPCHK(hipEventRecord(h->ev[2 * h->prof_n], st));
            int rc;
            if (gemv) {
                rc = B == 1 ? launch_gemv<1>(h, sc, st, B, L, mask) : B == 2 ? launch_gemv<2>(h, sc, st, B, L, mask) : launch_gemv<4>(h, sc, st, B, L, mask);
            } else {
                // a sparse pass has few bank tiles: give each workgroup fewer queries, so that more
                // workgroups share the pass and each one's k-loop is shorter
                int lqt = qt;
                while (lqt > 32 && (int64_t)L.ntiles * (Bp / lqt) < 128) lqt >>= 1;
                rc = mask.tags ? launch_mfma_any<true>(h, sc, st, Bp, lqt, L, k1, mask, B) : launch_mfma_any<false>(h, sc, st, Bp, lqt, L, k1, mask, B);
            }
            if (rc != MEM_OK) return rc;
            if (prof) {
                HIPCHK(hipEventRecord(h->ev[2 * h->prof_n + 1], st));
                int64_t rows = (int64_t)L.ntiles * TILE_ROWS;
                h->prof_rows[h->prof_n++] = rows;
            }
            if (li == plan.n - 1) {
                if (fused_tail) break;                              // the last selection runs inside the fused kernel below
                // the last selection refines a crowded band with exactly accumulated similarities
                with_store_type(h->dtype, [&](auto dt) {
                    hipLaunchKernelGGL(k_select_final<decltype(dt)::value>, dim3(B), dim3(1024), 0, st, surv, cnt, thr, (const float*)invq,
                                       counters, flags, k1, margin, mask.tags != nullptr, keep_of(k1), (const void*)h->store,
                                       (const float*)qf, (const double*)invq64, h->nkb);
                });
            } else {
                hipLaunchKernelGGL(k_select, dim3(B), dim3(1024), 0, st, surv, cnt, thr, (const float*)invq, counters, flags, k1, margin,
                                   mask.tags != nullptr, keep_of(k1));
            }
            LAUNCHCHK();
        }
        if (fused_tail) {
            const float* qs = (const float*)(h->q + (int64_t)stage * h->capacity);
            with_store_type(h->dtype, [&](auto dt) {
                hipLaunchKernelGGL(k_select_rescore_rerank<decltype(dt)::value>, dim3(B), dim3(1024), 0, st, surv, cnt, thr,
                                   (const float*)invq, counters, flags, k1, margin, mask.tags != nullptr, keep_of(k1),
                                   (const void*)h->store, (const float*)qf, (const double*)invq64, exact, h->nkb, exact_stride, qs, k2,
                                   (double)lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev, out_cand_sims_dev, eg);
            });
            LAUNCHCHK();
            return MEM_OK;
        }
    }
    if (h->N > 0) {
        // a query's candidates are split over several workgroups when there are few queries, so that the
        // gather occupies the whole device
        // (measured: 151 -> 102 us at B = 128, d = 4096; no gain at B = 256)
        int rsplit = 1;
        while (B <= 128 && rsplit < 8 && B * rsplit < 512) rsplit <<= 1;
        dim3 rgrid((unsigned)B, (unsigned)rsplit);
        with_store_type(h->dtype, [&](auto dt) {
            hipLaunchKernelGGL(k_rescore<decltype(dt)::value>, rgrid, dim3(1024), 0, st, (const void*)h->store, (const float*)qf,
                               (const double*)invq64, (const uint64_t*)surv, (const uint32_t*)cnt, exact, h->nkb, exact_stride);
        });
        LAUNCHCHK();
    }
    if (k1 <= 128) {                       // counting ranks is quadratic: measured faster than sorting up to here
        hipLaunchKernelGGL(k_rerank, dim3(B), dim3(RERANK_T), 0, st, (const uint64_t*)surv, (const uint32_t*)cnt, (const double*)exact,
                           (const float*)(h->q + (int64_t)stage * h->capacity), k1, k2, (double)lambda, out_ids_dev, out_scores_dev,
                           out_cand_ids_dev, out_cand_sims_dev, eg, exact_stride);
    } else {                               // larger pools: sorts instead of counting ranks
        int cap = 2;
        while (cap < keep_of(k1)) cap <<= 1;
        const size_t lds = rerank_big_lds(cap, k1, k2);
        static bool lds_set[MAX_DEVICES] = {};
        if (!lds_set[h->device]) {
            HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_rerank_big), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)rerank_big_lds(4096, BIG_K1_MAX, BIG_K1_MAX)));
            lds_set[h->device] = true;
        }
        hipLaunchKernelGGL(k_rerank_big, dim3(B), dim3(BIG_T), lds, st, (const uint64_t*)surv, (const uint32_t*)cnt,
                           (const double*)exact, exact_stride, (const float*)(h->q + (int64_t)stage * h->capacity), k1, k2,
                           (double)lambda, cap, out_ids_dev, out_scores_dev, out_cand_ids_dev, out_cand_sims_dev, eg);
    }
    LAUNCHCHK();
    return MEM_OK;
}

// the scratch area a handle was created with
static Scratch own_scratch(const evomem* h) { return Scratch{h->ws, h->w, keep_of(h->max_k1)}; }

extern "C" int mem_retrieve(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                            int32_t* out_ids_dev, float* out_scores_dev, int32_t* out_cand_ids_dev,
                            float* out_cand_sims_dev, void* hip_stream) {
    if (!h) return MEM_EINVAL;
    const EpsGreedy greedy{0, 0, 0, nullptr};
    return retrieve_impl(h, queries_dev, B, stage, k1, k2, lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev,
                         out_cand_sims_dev, hip_stream, greedy, Mask{nullptr, nullptr, nullptr}, own_scratch(h), h->max_B, h->max_k1);
}

// The library's own scratch area for mem_retrieve_static: one array per GPU, in that GPU's memory for
// as long as the library is loaded.  In host code the array's name only stands for the symbol; its
// device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static unsigned char* scratch_ptr[MAX_DEVICES] = {};

extern "C" int mem_retrieve_static(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                                   int32_t* out_ids_dev, float* out_scores_dev, int32_t* out_cand_ids_dev,
                                   float* out_cand_sims_dev, void* hip_stream) {
    if (!h) return MEM_EINVAL;
    if (h->nkb * KB > STATIC_MAX_D) return MEM_EINVAL;            // B and k1 are checked against their limits below
    int cur = -1;
    HIPCHK(hipGetDevice(&cur));
    if (cur != h->device) return MEM_ESTATE;
    if (!scratch_ptr[cur]) {                                      // first call on this device
        unsigned char* p = nullptr;
        HIPCHK(hipGetSymbolAddress(reinterpret_cast<void**>(&p), HIP_SYMBOL(scratch)));
        if (!p) return MEM_EHIP;
        // the counter block must start at zero; everything else is written before it is read in every call
        hipLaunchKernelGGL(k_clear_words, dim3(1), dim3(64), 0, static_cast<hipStream_t>(hip_stream),
                           reinterpret_cast<uint32_t*>(p + STATIC_W.counters), 64);
        LAUNCHCHK();
        scratch_ptr[cur] = p;
    }
    const EpsGreedy greedy{0, 0, 0, nullptr};
    return retrieve_impl(h, queries_dev, B, stage, k1, k2, lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev,
                         out_cand_sims_dev, hip_stream, greedy, Mask{nullptr, nullptr, nullptr},
                         Scratch{scratch_ptr[cur], STATIC_W, keep_of(STATIC_MAX_K1)}, STATIC_MAX_B, STATIC_MAX_K1);
}

extern "C" int mem_retrieve_exact(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                                  int32_t* out_ids_dev, float* out_scores_dev, int32_t* out_cand_ids_dev,
                                  float* out_cand_sims_dev, void* hip_stream) {
    if (!h) return MEM_EINVAL;
    const EpsGreedy greedy{0, 0, 0, nullptr};
    return retrieve_impl(h, queries_dev, B, stage, k1, k2, lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev,
                         out_cand_sims_dev, hip_stream, greedy, Mask{nullptr, nullptr, nullptr}, own_scratch(h), h->max_B, h->max_k1, true);
}

extern "C" int mem_retrieve_flags(evomem_t* h, uint32_t* out_flags_dev, int B, void* hip_stream) {
    if (!h || B < 0 || (B > 0 && !out_flags_dev)) return MEM_EINVAL;
    if (B == 0) return MEM_OK;
    if (!h->last_flags || B > h->last_B) return MEM_ESTATE;      // no retrieve yet, or a smaller one
    HIPCHK(hipMemcpyAsync(out_flags_dev, h->last_flags, sizeof(uint32_t) * (size_t)B, hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(hip_stream)));
    return MEM_OK;
}

extern "C" int mem_retrieve_eps(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                                float eps, uint64_t seed, uint64_t step, int32_t* out_ids_dev, float* out_scores_dev,
                                int32_t* out_cand_ids_dev, float* out_cand_sims_dev, unsigned char* out_explored_dev,
                                void* hip_stream) {
    if (!h) return MEM_EINVAL;
    if (!(eps >= 0.f && eps <= 1.f)) return MEM_EINVAL;
    const EpsGreedy eg{(uint64_t)((double)eps * 4294967296.0), seed, step, out_explored_dev};
    return retrieve_impl(h, queries_dev, B, stage, k1, k2, lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev,
                         out_cand_sims_dev, hip_stream, eg, Mask{nullptr, nullptr, nullptr}, own_scratch(h), h->max_B, h->max_k1);
}

extern "C" int mem_attach_tags(evomem_t* h, uint32_t* tags_dev) {
    if (!h || !tags_dev) return MEM_EINVAL;
    HIPCHK(hipMemset(tags_dev, 0, sizeof(uint32_t) * (size_t)h->capacity));
    h->tags = tags_dev;
    return MEM_OK;
}

extern "C" int mem_set_tags(evomem_t* h, int64_t first, int64_t n, const uint32_t* tags_dev, void* hip_stream) {
    if (!h || first < 0 || n < 0 || first + n > h->N) return MEM_EINVAL;
    if (!h->tags) return MEM_ESTATE;
    if (n == 0) return MEM_OK;
    if (!tags_dev) return MEM_EINVAL;
    HIPCHK(hipMemcpyAsync(h->tags + first, tags_dev, sizeof(uint32_t) * (size_t)n, hipMemcpyDeviceToDevice,
                          static_cast<hipStream_t>(hip_stream)));
    return MEM_OK;
}

extern "C" int mem_retrieve_masked(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                                   const uint32_t* allow_types_dev, const uint32_t* exclude_group_dev,
                                   int32_t* out_ids_dev, float* out_scores_dev, int32_t* out_cand_ids_dev,
                                   float* out_cand_sims_dev, void* hip_stream) {
    if (!h) return MEM_EINVAL;
    if (!h->tags) return MEM_ESTATE;
    if (B > 0 && (!allow_types_dev || !exclude_group_dev)) return MEM_EINVAL;
    const EpsGreedy greedy{0, 0, 0, nullptr};
    return retrieve_impl(h, queries_dev, B, stage, k1, k2, lambda, out_ids_dev, out_scores_dev, out_cand_ids_dev,
                         out_cand_sims_dev, hip_stream, greedy, Mask{h->tags, allow_types_dev, exclude_group_dev}, own_scratch(h),
                         h->max_B, h->max_k1);
}

extern "C" int mem_select_by_q(evomem_t* h, const int32_t* set_ids_dev, int64_t n_ids, const int64_t* set_offsets_dev,
                               int G, int stage, float eps, uint64_t seed, uint64_t step, int32_t* out_ids_dev,
                               float* out_q_dev, unsigned char* out_explored_dev, void* hip_stream) {
    if (!h || G < 0 || n_ids < 0 || (stage != 0 && stage != 1) || !(eps >= 0.f && eps <= 1.f)) return MEM_EINVAL;
    if (G == 0) return MEM_OK;
    if (!set_offsets_dev || !out_ids_dev || !out_q_dev || (n_ids > 0 && !set_ids_dev)) return MEM_EINVAL;
    const EpsGreedy eg{(uint64_t)((double)eps * 4294967296.0), seed, step, out_explored_dev};
    hipLaunchKernelGGL(k_select_by_q, dim3((unsigned)G), dim3(SP_LANES), 0, static_cast<hipStream_t>(hip_stream),
                       set_ids_dev, n_ids, set_offsets_dev, (const float*)(h->q + (int64_t)stage * h->capacity), h->N, eg,
                       out_ids_dev, out_q_dev, (uint32_t*)(h->ws + h->w.counters));
    LAUNCHCHK();
    return MEM_OK;
}

extern "C" int mem_update_q(evomem_t* h, const int32_t* ids_dev, int64_t M, int stage, const float* rewards_dev,
                            float alpha, void* hip_stream) {
    if (!h || M < 0 || (stage != 0 && stage != 1) || !(alpha > 0.f && alpha <= 1.f)) return MEM_EINVAL;
    if (M == 0) return MEM_OK;
    if (!ids_dev || !rewards_dev) return MEM_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint32_t* counters = (uint32_t*)(h->ws + h->w.counters);
    static bool lds_set[MAX_DEVICES] = {};          // the kernel's LDS list can exceed the default 64 KB limit
    if (!lds_set[h->device]) {
        HIPCHK(hipFuncSetAttribute(reinterpret_cast<const void*>(k_update_q), hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (UPD_CHUNK + UPD_PAD) * 8));
        lds_set[h->device] = true;
    }
    for (int64_t off = 0; off < M; off += UPD_CHUNK) {
        int m = (int)(M - off < UPD_CHUNK ? M - off : UPD_CHUNK);
        const int lg = upd_log2_buckets(m);
        int npad = 2;                      // a bucket may receive every pair of the launch
        while (npad < m) npad <<= 1;
        hipLaunchKernelGGL(k_update_q, dim3(1u << lg), dim3(1024), (size_t)(npad + UPD_PAD) * 8, st, ids_dev + off, rewards_dev + off, m,
                           h->q + (int64_t)stage * h->capacity, h->N, alpha, counters, lg);
        LAUNCHCHK();
    }
    return MEM_OK;
}
