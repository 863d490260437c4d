/*
 * evomem -- value-driven memory retrieval on one MI355X (gfx950), C ABI.
 *
 * The library implements the retrieval policy mu of Sec. 3.2 of the paper ("Memory Architecture
 * and Value-Driven Retrieval") over a growing bank of embedded memory items (Sec. 3.1, memory
 * growth rule):
 *
 *   mem_append    M_{t+1} <- M_t u {...}: add entries to the bank (Sec. 3.1, memory update rule).
 *   mem_retrieve  dense recall of a top-k1 candidate pool by cosine similarity, then the
 *                 stage-specific value filter down to the final k2 items (Sec. 3.2; k1 is the
 *                 paper's K, k2 the paper's final retrieval count N).
 *   mem_update_q  unified Monte-Carlo value update Q <- Q + alpha (r - Q) for the given ids
 *                 (Sec. 3.2, Eq. "unified update"; App. A, bandit-style update).
 *
 * Conventions
 *   - Every `*_dev` pointer is DEVICE memory owned by the caller (for instance a torch tensor's
 *     data_ptr) and must stay valid until mem_destroy.  The library owns only its host handle and
 *     a few HIP events.  Pointers without the suffix are HOST memory.
 *   - `hip_stream` is a hipStream_t passed as void*; NULL is the default stream.  Calls on one
 *     stream are ordered; using one handle from several streams at once is not supported, and the
 *     library's calls must come from one host thread at a time (it keeps small per-device caches,
 *     such as how many workgroups of a kernel the device holds, without locks).
 *   - No call synchronises with the host except those documented to do so.
 *   - mem_retrieve (and its variants), mem_update_q, mem_retrieve_flags, mem_shape_rewards and
 *     mem_select_by_q only launch kernels and device-to-device copies on the given stream: once a first
 *     call of each has run on the device (it does per-device set-up), they can be recorded into a HIP
 *     graph and replayed.  mem_append cannot: it counts the bank's entries on the host.
 *   - Entry ids are dense int32: 0,1,2,... in append order, never reused (the bank only grows).
 *   - Similarity is the cosine between the STORED vectors: rows and queries are rounded to the
 *     bank's element type (round-to-nearest-even) first; accumulation is fp32 or wider and the
 *     similarities that reach the value filter are accumulated in fp64.
 *   - Order rule in both selections: larger value first, lower id first among equal values.
 *   - Value filter: score = (1-lambda) z(sim) + lambda z(Q_stage), z being the z-score over the
 *     query's own candidate pool (population standard deviation, denominator std + 1e-6).
 *     lambda = 0 ranks by similarity alone, lambda = 1 by the stage's Q alone.
 *   - All functions return a mem_status; nothing throws or aborts.  NaN, infinite or zero-norm rows,
 *     queries and Q values are not checked on the hot path: which items such a call returns is
 *     unspecified, but it is well formed (every id is -1 or an entry of the bank, none twice in a
 *     pool) and later calls are unaffected.
 */
#ifndef EVOMEM_H
#define EVOMEM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct evomem evomem_t; /* opaque host handle */

enum mem_status {
    MEM_OK = 0,
    MEM_EINVAL = 1,     /* bad argument (null pointer, bad enum, size out of range, ...) */
    MEM_ECAPACITY = 2,  /* append would exceed the capacity given at creation; nothing is appended */
    MEM_EWORKSPACE = 3, /* workspace smaller than mem_workspace_bytes() for the stated maxima */
    MEM_EHIP = 4,       /* a HIP runtime call failed */
    MEM_ESTATE = 5      /* handle unusable (e.g. created for another device) */
};
enum mem_dtype { MEM_F32 = 0, MEM_BF16 = 1, MEM_F16 = 2 }; /* storage element type */
enum mem_stage { MEM_STAGE_DRAFT = 0, MEM_STAGE_REFINE = 1 }; /* Q_1 / Q_2 of Sec. 3.2 */

#define MEM_MAX_K1 2048  /* largest candidate pool (Sec. 4.4 studies pools of 3x to 30x the final count) */
#define MEM_MAX_B 4096   /* largest query batch per call */

/* Bytes the caller must allocate for the embedding store (tiled layout, padded), for given
 * dimension (multiple of 8, 8..16384), element type and capacity (entries, 1 .. 2^31-257).
 * Returns 0 on bad arguments. */
size_t mem_store_bytes(int d, int dtype, int64_t capacity);

/* Bytes of scratch the caller must allocate for calls with B <= max_B and k1 <= max_k1.
 * Returns 0 on bad arguments. */
size_t mem_workspace_bytes(int d, int dtype, int64_t capacity, int max_B, int max_k1);

/*
 * Create an empty bank (Sec. 3.1: M_0 is whatever the caller appends first).  Touches no device
 * memory except a clear of two counters at the head of the workspace, which it waits for.
 *   store_dev      mem_store_bytes() bytes, 256-byte aligned
 *   invnorm_dev    float[capacity rounded up to a multiple of 256]
 *   q_dev          float[2][capacity]: row 0 = drafting values Q_1, row 1 = refining values Q_2
 *   workspace_dev  mem_workspace_bytes() bytes, 256-byte aligned
 *   device         HIP device ordinal the buffers live on, 0..15; it becomes the calling thread's current device
 * Errors: MEM_EINVAL, MEM_EWORKSPACE, MEM_EHIP.
 */
int mem_create(evomem_t** out, int d, int dtype, int64_t capacity,
               void* store_dev, float* invnorm_dev, float* q_dev,
               void* workspace_dev, size_t workspace_bytes, int max_B, int max_k1, int device);

/*
 * Append n entries (Sec. 3.1, memory update rule).  emb_dev: float[n][d] row-major, any norm.
 * q0_*_dev: float[n] initial values for the two tables, or NULL for 0 (App. A only requires Q_0
 * inside the reward range).  *first_id_out (host, may be NULL) receives the id of the first new
 * entry; the rest follow consecutively.  n = 0 is a no-op.
 * Errors: MEM_EINVAL, MEM_ECAPACITY (bank unchanged), MEM_EHIP.
 */
int mem_append(evomem_t* h, const float* emb_dev, int64_t n,
               const float* q0_draft_dev, const float* q0_refine_dev,
               int64_t* first_id_out, void* hip_stream);

/*
 * Retrieve for B queries (Sec. 3.2: top-K pool by dense retrieval, then filter by Q_stage to the
 * final items).  queries_dev: float[B][d].  With N entries in the bank, k1_eff = min(k1, N) and
 * k2_eff = min(k2, k1_eff).
 *   out_ids_dev     int32[B][k2]   final items, best first; unused slots -1
 *   out_scores_dev  float[B][k2]   their scores; unused slots -inf
 *   out_cand_ids_dev / out_cand_sims_dev   int32/float [B][k1] the candidate pool ordered by
 *                   (similarity desc, id asc), or NULL (both or neither); unused slots -1 / -inf
 * B = 0 is a no-op.  Errors: MEM_EINVAL (null pointers, stage, k1 < 1, k2 < 1, k2 > k1,
 * k1 > max_k1, B > max_B, lambda outside [0,1] or NaN), MEM_EHIP.
 */
int mem_retrieve(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2,
                 float lambda, int32_t* out_ids_dev, float* out_scores_dev,
                 int32_t* out_cand_ids_dev, float* out_cand_sims_dev, void* hip_stream);

/*
 * mem_retrieve by exhaustive selection: the same arguments and the same results, reached without
 * thresholds or scan passes -- the similarity of EVERY entry to every query is accumulated in fp64
 * (rounded to fp32 for the selection: entries whose similarities differ by less than 6e-8 rank by id) and
 * the pool is selected range by range, so no list can overflow whatever the bank holds.  It reads the
 * bank once per QUERY instead of once per batch (1M x 1024 bf16 entries: about 1 ms per query), so it is
 * the call for the queries that mem_retrieve_flags reports, and an on-device cross-check of mem_retrieve.
 * Greedy selection only.  Errors: as mem_retrieve.
 */
int mem_retrieve_exact(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2,
                       float lambda, int32_t* out_ids_dev, float* out_scores_dev,
                       int32_t* out_cand_ids_dev, float* out_cand_sims_dev, void* hip_stream);

/*
 * Per-query status of the latest retrieve call of any kind on this handle (enqueued on the same stream,
 * or ordered after it): copies B words to out_flags_dev (uint32[B]) on the stream, without synchronising.
 * Bit 0 (MEM_FLAG_OVERFLOW): during some scan pass more than 8192 rows of the bank reached the query's
 * running threshold (the k1-th best similarity seen so far, minus a rounding margin) -- a mass of
 * near-duplicates of the pool's last members.  The rows beyond 8192 were not kept, so the pool of such a
 * query may miss members whose similarity ties with its last ones; every other query of the call is
 * exact, and mem_retrieve_exact answers the flagged ones exactly.  Errors: MEM_EINVAL, MEM_ESTATE (no retrieve yet, or B larger than that call's), MEM_EHIP.
 */
#define MEM_FLAG_OVERFLOW 1u
int mem_retrieve_flags(evomem_t* h, uint32_t* out_flags_dev, int B, void* hip_stream);

/*
 * mem_retrieve for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc) and so cannot size and bring a workspace of their
 * own: the same call, same arguments, same results bit for bit, but every intermediate result lives
 * in an array that is part of the library itself (5.3 MB per GPU, held while the library is loaded)
 * instead of the workspace given to mem_create, which this call never touches.  It allocates nothing
 * on the device or through any allocating routine.
 * Limits: B <= 64, k1 <= 256, d <= 2048 (after padding to a multiple of 64); beyond them MEM_EINVAL.
 * The handle's device must be the current device (MEM_ESTATE otherwise).  The first call on a device
 * looks the array's address up and enqueues a small kernel that clears its counter block.
 * All handles and streams of a process share the one array of a GPU: calls that overlap on one GPU
 * race; calls ordered on one stream (or otherwise serialised) do not.  Queries whose survivor list
 * overflows are counted inside the array, not in the handle's mem_counters (mem_retrieve_flags reports them).
 */
int mem_retrieve_static(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2,
                        float lambda, int32_t* out_ids_dev, float* out_scores_dev,
                        int32_t* out_cand_ids_dev, float* out_cand_sims_dev, void* hip_stream);

/*
 * Retrieve with epsilon-greedy selection of the final items (Sec. 3.3, Stage 1: the drafting
 * context is drawn from the pool C(x) by an epsilon-greedy policy over Q_1; Sec. 4.4 uses the same
 * policy for both stages).  The pool and the scores are those of mem_retrieve; the k2 slots are
 * filled in order: with probability eps a slot takes a uniformly random member of the pool that is
 * not chosen yet, otherwise the best one not chosen yet (score desc, id asc).  eps = 0 gives
 * exactly mem_retrieve's result.
 * The draws are a pure function of (seed, step, query row, slot): Philox-4x32 with 10 rounds, key =
 * seed (low word, high word), counter = (step low, step high, query row, slot).  Output word 0
 * decides: explore iff word0 < floor(eps * 2^32), compared as 64-bit integers.  Output word 1 picks:
 * index floor(word1 * remaining / 2^32) among the members not chosen yet, in greedy order.  A caller
 * that passes its iteration counter as `step` can therefore replay any call.
 *   out_scores_dev    the chosen items' scores (not sorted: slot order)
 *   out_explored_dev  uint8[B][k2], 1 where the slot was filled by the random branch; may be NULL
 * Errors: as mem_retrieve, and MEM_EINVAL for eps outside [0,1] or NaN.
 */
int mem_retrieve_eps(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2,
                     float lambda, float eps, uint64_t seed, uint64_t step,
                     int32_t* out_ids_dev, float* out_scores_dev,
                     int32_t* out_cand_ids_dev, float* out_cand_sims_dev,
                     unsigned char* out_explored_dev, void* hip_stream);

/*
 * Typed / masked retrieval.  The bank of Sec. 3.2 holds items of several types (kernel code with
 * its outcome, API templates, generation traces, summarised experience), and the generalisation
 * study of Sec. 4.3 leaves the entries of held-out operators out of retrieval.  Every entry carries
 * a 32-bit tag: type = tag & 0xff (types 0..31 can be retrieved), group = tag >> 8 (for instance the
 * operator the entry stems from).
 *   mem_attach_tags      hands the library a caller-owned device array uint32[capacity] for the tags;
 *                        it is zero-filled (type 0, group 0) synchronously.  Needed once, before the
 *                        two calls below (they return MEM_ESTATE otherwise).
 *   mem_set_tags         copies n tags for entries first .. first+n-1 (which must exist) on the stream.
 *   mem_retrieve_masked  as mem_retrieve, but query b only sees entries whose type bit is set in
 *                        allow_types_dev[b] and whose group differs from exclude_group_dev[b]
 *                        (0xffffffff excludes nothing): the pool is the top-k1 among those, and
 *                        k1_eff = min(k1, number of such entries).  Both arrays are uint32[B].
 * A query whose accepted entries are rare in the bank is still answered exactly, but slowly: the
 * scan's threshold can only be as tight as the accepted entries of the sparsest pass allow.
 */
int mem_attach_tags(evomem_t* h, uint32_t* tags_dev);
int mem_set_tags(evomem_t* h, int64_t first, int64_t n, const uint32_t* tags_dev, void* hip_stream);
int mem_retrieve_masked(evomem_t* h, const float* queries_dev, int B, int stage, int k1, int k2, float lambda,
                        const uint32_t* allow_types_dev, const uint32_t* exclude_group_dev,
                        int32_t* out_ids_dev, float* out_scores_dev,
                        int32_t* out_cand_ids_dev, float* out_cand_sims_dev, void* hip_stream);

/*
 * Value update (Sec. 3.2, Eq. "unified update"): for j = 0..M-1 in array order,
 * Q_stage[ids[j]] <- Q + alpha (rewards[j] - Q), each operation rounded to fp32 (no fused
 * multiply-add).  An id that occurs several times receives its rewards one after another in array
 * order (the recursion unrolled in App. A).  Every other entry, and the other stage's table, is
 * left bit-for-bit unchanged.  Ids outside [0, N) are skipped and counted.  No floating-point
 * atomics: one writer per distinct id.  M = 0 is a no-op.
 * Errors: MEM_EINVAL (null pointers, stage, M < 0, alpha outside (0,1] or NaN), MEM_EHIP.
 */
int mem_update_q(evomem_t* h, const int32_t* ids_dev, int64_t M, int stage,
                 const float* rewards_dev, float alpha, void* hip_stream);

/* Number of entries in the bank (host-side counter). */
int mem_size(const evomem_t* h, int64_t* n_out);

/* Copy Q_stage[first .. first+n) into dst_dev (float[n]).  For tests and export. */
int mem_read_q(evomem_t* h, int stage, int64_t first, int64_t n, float* dst_dev, void* hip_stream);

/*
 * Rewards of the two stages from verifier outcomes, ready for mem_update_q.
 *   stage 0 (Sec. 3.3, cold-start drafting): +1 if feasible_dev[j] != 0, else -1; the latency
 *           arrays are not read and may be NULL.
 *   stage 1 (Sec. 3.4, continual refining): -1 if infeasible, else
 *           tanh(log best_latency_dev[j] - log latency_dev[j])  (App. A: tanh(log rho)); latencies > 0.
 * normalise != 0 applies the online normalisation of Sec. 3.4 / App. A in array order: sample j
 * becomes (r_j - mu) / max(sigma, sigma_min), then is clipped to [-clip, clip] if clip > 0, where
 * mu and sigma are the running mean and population deviation of all raw rewards of this stage seen
 * BEFORE sample j (in earlier calls and earlier in this batch; before the first sample mu = 0 and
 * sigma = 0).  The statistics are kept per stage in the workspace in fp64.
 * rewards_out_dev: float[M].  M = 0 is a no-op.
 * Errors: MEM_EINVAL (null pointers, stage, sigma_min <= 0 with normalise, clip < 0 or NaN), MEM_EHIP.
 */
int mem_shape_rewards(evomem_t* h, int stage, const unsigned char* feasible_dev, const float* latency_dev,
                      const float* best_latency_dev, int64_t M, int normalise, float sigma_min, float clip,
                      float* rewards_out_dev, void* hip_stream);

/* Synchronises the device.  Running statistics of stage's raw rewards: how many, their mean and
 * population deviation (App. A, running statistics). */
int mem_reward_stats(evomem_t* h, int stage, double* count, double* mean, double* sigma);

/* Forget the running statistics of a stage (asynchronous on the stream). */
int mem_reward_stats_reset(evomem_t* h, int stage, void* hip_stream);

/*
 * Start-point selection (Sec. 3.4: among the start points P(x) available for a task, one is
 * selected using Q_2; Sec. 4.4: by the same epsilon-greedy policy as the contexts).  G sets at once:
 * set g is set_ids_dev[set_offsets_dev[g] .. set_offsets_dev[g+1]) (int32 ids, int64 offsets, G + 1
 * of them, non-decreasing, within [0, n_ids]; offsets outside that range are clamped to it).  Ids
 * outside [0, size) are not members of their set; they are counted in mem_counters' skipped ids.
 *   out_ids_dev       int32[G]  the member with the largest value in the stage's table, the lower id
 *                     among equal values (-0 equals +0, a NaN value counts as -inf); -1 for a set
 *                     without members
 *   out_q_dev         float[G]  that entry's value as stored; 0 for a set without members
 *   out_explored_dev  uint8[G]  1 where the random branch chose; may be NULL
 * With probability eps a set takes, instead of its best member, the member at a uniformly random
 * position (a repeated id is as many times more likely).  The draw is Philox-4x32 with 10 rounds,
 * key = seed, counter = (step low, step high, g, 0xffffffff) -- the last word keeps it apart from
 * the draws of mem_retrieve_eps' slots under the same seed and step.  Word 0 decides (explore iff
 * word0 < floor(eps * 2^32)), word 1 picks position floor(word1 * members / 2^32) in array order.
 * G = 0 is a no-op.  Errors: MEM_EINVAL (null pointers, G < 0, n_ids < 0, stage, eps outside [0,1]
 * or NaN), MEM_EHIP.
 */
int mem_select_by_q(evomem_t* h, const int32_t* set_ids_dev, int64_t n_ids, const int64_t* set_offsets_dev,
                    int G, int stage, float eps, uint64_t seed, uint64_t step, int32_t* out_ids_dev,
                    float* out_q_dev, unsigned char* out_explored_dev, void* hip_stream);

/*
 * Re-use of a bank across runs (Sec. 4.3 transfers a memory built on one set of tasks to others).
 * Every buffer of a bank belongs to the caller, so saving a bank is copying the caller's store,
 * inverse-norm, value-table (and tag) buffers together with mem_size().  To continue from such a
 * copy: create a handle over buffers that already hold it (same d, dtype and capacity, so that the
 * store layout is the same) and declare with mem_restore how many entries they hold.  Nothing is
 * read or checked; n entries are simply taken to exist.  Errors: MEM_EINVAL (n < 0), MEM_ECAPACITY.
 */
int mem_restore(evomem_t* h, int64_t n);

/* Copy stored rows first .. first+n, widened to fp32 and un-tiled, into dst_dev (float[n][d]). */
int mem_read_rows(evomem_t* h, int64_t first, int64_t n, float* dst_dev, void* hip_stream);

/* Synchronises the device.  *skipped_ids: ids outside the bank that mem_update_q and mem_select_by_q
 * have skipped so far; *overflows: queries whose survivor list overflowed during some retrieve so far
 * (their pool may then be inexact; mem_retrieve_flags names them per call, without synchronising). */
int mem_counters(evomem_t* h, int64_t* skipped_ids, int64_t* overflows);

/* Per-kernel timing with HIP events on the call's stream (off by default).  While on, every
 * launch of the similarity-scan kernel is bracketed by two events (at most 4096 launches are kept
 * between reads; switching off and on again keeps what was recorded, so a caller can time a
 * sample of its calls -- each event costs a few microseconds of idle time around the launch).  mem_profile_read synchronises the device and writes, for up to `capacity`
 * launches recorded since the last read, in launch order: ms_out[i] the duration in milliseconds,
 * rows_out[i] the number of bank rows that launch scanned; *n_out is how many were written. */
int mem_profile_enable(evomem_t* h, int on);
int mem_profile_read(evomem_t* h, int capacity, int* n_out, float* ms_out, int64_t* rows_out);

/* Measurement aid: one read-only pass over the rows the bank holds (whole 256-row tiles), every byte
 * loaded once and XOR-folded into *checksum_dev (uint32, the caller clears it); *bytes_out (host, may be
 * NULL) receives the number of bytes read.  The similarity scan of a retrieve has to read the same bytes,
 * so this launch's duration is the floor that the machine at hand sets for it. */
int mem_read_probe(evomem_t* h, uint32_t* checksum_dev, int64_t* bytes_out, void* hip_stream);

/* Host only, for tests of the scan plan: the passes a retrieve with pool size k1 makes over a bank of
 * N entries, sparsest first.  Pass i scans the 256-row tiles t = u * stride[i] (u = 0,1,...) below
 * ceil(N/256), leaving out those with u % rho[i] == 0 when rho[i] > 0 (a sparser pass owns them);
 * ntiles[i] is their number.  Returns the number of passes (at most max_levels are written), or -1
 * on bad arguments. */
int mem_plan_levels(int64_t N, int k1, int* stride, int* rho, int* ntiles, int max_levels);

const char* mem_strerror(int status);
int mem_destroy(evomem_t* h);

#ifdef __cplusplus
}
#endif
#endif /* EVOMEM_H */
