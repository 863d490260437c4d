/*
 * A plain C caller of the library's C ABI: no Python, no torch.  It allocates device memory with the
 * HIP runtime, builds a small bank from the rows in an input file, retrieves, updates the values of
 * the returned items and prints everything as text.  tests/test_gpu_abi_client.py builds it with
 * gcc, runs it on the GPU and checks what it prints against the CPU oracle.
 *
 * Input file (little endian): int32 N, d, B, k1, k2, stage; float lambda, alpha;
 * float rows[N][d]; float queries[B][d]; float q0[2][N]; float rewards[B*k2].
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "evomem.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); return 2; } } while (0)
#define CHECK_MEM(x) do { int s_ = (x); if (s_ != MEM_OK) { fprintf(stderr, "%s: %s\n", #x, mem_strerror(s_)); return 3; } } while (0)

static void* upload(const void* host, size_t bytes) {
    void* dev = NULL;
    if (hipMalloc(&dev, bytes ? bytes : 16) != hipSuccess) return NULL;
    if (bytes && hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice) != hipSuccess) return NULL;
    return dev;
}

int main(int argc, char** argv) {
    if (argc < 2) { fprintf(stderr, "usage: %s input.bin\n", argv[0]); return 1; }
    FILE* f = fopen(argv[1], "rb");
    if (!f) { perror("input"); return 1; }
    int32_t hdr[6];
    float par[2];
    if (fread(hdr, 4, 6, f) != 6 || fread(par, 4, 2, f) != 2) return 1;
    const int N = hdr[0], d = hdr[1], B = hdr[2], k1 = hdr[3], k2 = hdr[4], stage = hdr[5];
    const float lambda = par[0], alpha = par[1];
    float* rows = malloc(sizeof(float) * (size_t)N * d);
    float* queries = malloc(sizeof(float) * (size_t)B * d);
    float* q0 = malloc(sizeof(float) * 2 * (size_t)N);
    float* rewards = malloc(sizeof(float) * (size_t)B * k2);
    if (fread(rows, 4, (size_t)N * d, f) != (size_t)N * d || fread(queries, 4, (size_t)B * d, f) != (size_t)B * d ||
        fread(q0, 4, 2 * (size_t)N, f) != 2 * (size_t)N || fread(rewards, 4, (size_t)B * k2, f) != (size_t)B * k2) return 1;
    fclose(f);

    CHECK_HIP(hipSetDevice(0));
    const int64_t capacity = N;
    const size_t store_bytes = mem_store_bytes(d, MEM_F32, capacity);
    const size_t ws_bytes = mem_workspace_bytes(d, MEM_F32, capacity, B, k1);
    void *store = NULL, *ws = NULL;
    float *invnorm = NULL, *qtab = NULL;
    CHECK_HIP(hipMalloc(&store, store_bytes));
    CHECK_HIP(hipMalloc(&ws, ws_bytes));
    CHECK_HIP(hipMalloc((void**)&invnorm, sizeof(float) * (size_t)((capacity + 255) / 256 * 256)));
    CHECK_HIP(hipMalloc((void**)&qtab, sizeof(float) * 2 * (size_t)capacity));
    evomem_t* h = NULL;
    CHECK_MEM(mem_create(&h, d, MEM_F32, capacity, store, invnorm, qtab, ws, ws_bytes, B, k1, 0));

    /* append in two pieces, with initial values for both tables */
    const int n1 = N / 3;
    float* rows_dev = upload(rows, sizeof(float) * (size_t)N * d);
    float* q0a = upload(q0, sizeof(float) * (size_t)N);
    float* q0b = upload(q0 + N, sizeof(float) * (size_t)N);
    if (!rows_dev || !q0a || !q0b) return 2;
    int64_t first = -1;
    CHECK_MEM(mem_append(h, rows_dev, n1, q0a, q0b, &first, NULL));
    if (first != 0) return 4;
    CHECK_MEM(mem_append(h, rows_dev + (size_t)n1 * d, N - n1, q0a + n1, q0b + n1, &first, NULL));
    if (first != n1) return 4;
    int64_t size = 0;
    CHECK_MEM(mem_size(h, &size));
    printf("size %lld\n", (long long)size);

    float* queries_dev = upload(queries, sizeof(float) * (size_t)B * d);
    int32_t *ids_dev = NULL, *cand_dev = NULL;
    float *sc_dev = NULL, *csim_dev = NULL;
    CHECK_HIP(hipMalloc((void**)&ids_dev, sizeof(int32_t) * (size_t)B * k2));
    CHECK_HIP(hipMalloc((void**)&sc_dev, sizeof(float) * (size_t)B * k2));
    CHECK_HIP(hipMalloc((void**)&cand_dev, sizeof(int32_t) * (size_t)B * k1));
    CHECK_HIP(hipMalloc((void**)&csim_dev, sizeof(float) * (size_t)B * k1));
    CHECK_MEM(mem_retrieve(h, queries_dev, B, stage, k1, k2, lambda, ids_dev, sc_dev, cand_dev, csim_dev, NULL));
    float* rewards_dev = upload(rewards, sizeof(float) * (size_t)B * k2);
    CHECK_MEM(mem_update_q(h, ids_dev, (int64_t)B * k2, stage, rewards_dev, alpha, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    int32_t* ids = malloc(sizeof(int32_t) * (size_t)B * k2);
    float* sc = malloc(sizeof(float) * (size_t)B * k2);
    int32_t* cand = malloc(sizeof(int32_t) * (size_t)B * k1);
    float* csim = malloc(sizeof(float) * (size_t)B * k1);
    CHECK_HIP(hipMemcpy(csim, csim_dev, sizeof(float) * (size_t)B * k1, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(ids, ids_dev, sizeof(int32_t) * (size_t)B * k2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(sc, sc_dev, sizeof(float) * (size_t)B * k2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(cand, cand_dev, sizeof(int32_t) * (size_t)B * k1, hipMemcpyDeviceToHost));
    for (int b = 0; b < B; ++b) {
        printf("ids %d", b);
        for (int j = 0; j < k2; ++j) printf(" %d", ids[b * k2 + j]);
        printf("\nscores %d", b);
        for (int j = 0; j < k2; ++j) printf(" %.9g", sc[b * k2 + j]);
        printf("\ncand %d", b);
        for (int j = 0; j < k1; ++j) printf(" %d", cand[b * k1 + j]);
        printf("\ncsim %d", b);
        for (int j = 0; j < k1; ++j) printf(" %.9g", csim[b * k1 + j]);
        printf("\n");
    }
    /* both value tables after the update, as bit patterns */
    float* qout_dev = NULL;
    CHECK_HIP(hipMalloc((void**)&qout_dev, sizeof(float) * (size_t)N));
    uint32_t* qout = malloc(sizeof(uint32_t) * (size_t)N);
    for (int s = 0; s < 2; ++s) {
        CHECK_MEM(mem_read_q(h, s, 0, N, qout_dev, NULL));
        CHECK_HIP(hipMemcpy(qout, qout_dev, sizeof(float) * (size_t)N, hipMemcpyDeviceToHost));
        printf("q %d", s);
        for (int i = 0; i < N; ++i) printf(" %08x", qout[i]);
        printf("\n");
    }
    int64_t skipped = -1, overflows = -1;
    CHECK_MEM(mem_counters(h, &skipped, &overflows));
    printf("counters %lld %lld\n", (long long)skipped, (long long)overflows);
    /* argument errors come back as status codes */
    printf("einval %d\n", mem_retrieve(h, queries_dev, B, 7, k1, k2, lambda, ids_dev, sc_dev, NULL, NULL, NULL));
    CHECK_MEM(mem_destroy(h));
    printf("done\n");
    return 0;
}
