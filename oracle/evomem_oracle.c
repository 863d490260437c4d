/*
 * CPU oracle for value-driven memory retrieval (Sec. 3.2 of the paper) -- TEST INFRASTRUCTURE.
 *
 * Plain, slow, fp64, by-the-definition code.  It exists only so that tests, the smoke check and
 * the benchmark's CPU-baseline leg can compare the GPU library against it.  It shares no code,
 * header, table or helper with the GPU library, and nothing in the product path may call it.
 *
 * What it computes, in the paper's order (Sec. 3.2):
 *   1. dense recall: cosine similarity of a query against every stored entry, keep the K best
 *      (the "top-K candidate pool");
 *   2. value filter: re-rank the pool with the stage's Q values and keep the final N items;
 *   3. the unified Monte-Carlo value update Q <- Q + alpha (r - Q) for every id handed in
 *      (Eq. "unified update" of Sec. 3.2; App. A, bandit-style update).
 *
 * Readings where the paper gives no formula (each is pinned by a test on invariants):
 *   - similarity is the cosine of the *stored* (rounded to the bank's element type) vectors,
 *     queries being rounded to the same type first;
 *   - ties are broken towards the lower id, in both selections;
 *   - the re-rank score is (1-lam)*z(sim) + lam*z(Q), z being the z-score over the query's own
 *     candidate pool with population standard deviation and denominator (std + 1e-6);
 *   - duplicate ids in one update batch are applied one after another in array order, which is
 *     what the unrolled recursion in the proof of the constant-step-size lemma (App. A) describes.
 *
 * Pins: tests/test_oracle_pins.py (brute force, closed forms, invariants, library cross-checks).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };

/* ---------- element rounding: fp32 -> bank element type -> fp32, round-to-nearest-even ---------- */

static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

/* bfloat16 keeps the top 16 bits of the fp32 pattern; RNE on the dropped 16 bits. */
static float round_bf16(float x) {
    uint32_t u = float_to_bits(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return bits_to_float((u | 0x00400000u) & 0xffff0000u); /* NaN */
    uint32_t dropped = u & 0xffffu, keep = u >> 16;
    if (dropped > 0x8000u || (dropped == 0x8000u && (keep & 1u))) keep += 1; /* may carry into inf: correct */
    return bits_to_float(keep << 16);
}

/* IEEE binary16: 5 exponent bits (bias 15), 10 fraction bits, gradual underflow.  Done in exact
 * arithmetic: scale so that one unit in the last place of the target is 1.0, round to an integer
 * with ties-to-even, scale back. */
static float round_f16(float x) {
    if (isnan(x) || isinf(x) || x == 0.0f) return x;
    double a = fabs((double)x);
    int e;
    (void)frexp(a, &e);            /* a = m * 2^e, m in [0.5,1) -> exponent of leading bit is e-1 */
    int lead = e - 1;
    if (lead < -14) lead = -14;    /* subnormal range shares the ulp of the smallest normal */
    double ulp = ldexp(1.0, lead - 10);
    double q = a / ulp;            /* exact: power-of-two scaling */
    double fl = floor(q), frac = q - fl;
    if (frac > 0.5 || (frac == 0.5 && fmod(fl, 2.0) == 1.0)) fl += 1.0;
    double r = fl * ulp;
    if (r >= 65520.0) r = INFINITY; /* 65504 is the largest finite value; halfway point rounds up */
    return (float)(x < 0 ? -r : r);
}

/* out[i] = value the bank would hold for in[i], widened back to fp32 (exact). */
int orc_round_to_store(const float* in, int64_t count, int dtype, float* out) {
    if (dtype != ORC_F32 && dtype != ORC_BF16 && dtype != ORC_F16) return 1;
    for (int64_t i = 0; i < count; ++i)
        out[i] = dtype == ORC_F32 ? in[i] : dtype == ORC_BF16 ? round_bf16(in[i]) : round_f16(in[i]);
    return 0;
}

/* ---------- step 1: dense recall ---------- */

typedef struct { double sim; int32_t id; } pair_t;

/* sim descending, then id ascending */
static int pair_cmp(const void* pa, const void* pb) {
    const pair_t* a = (const pair_t*)pa; const pair_t* b = (const pair_t*)pb;
    if (a->sim > b->sim) return -1;
    if (a->sim < b->sim) return 1;
    return (a->id > b->id) - (a->id < b->id);
}

static double inv_norm(const float* v, int d) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += (double)v[i] * (double)v[i];
    return 1.0 / sqrt(ss);
}

/*
 * store   [N][d]  stored (already rounded, widened) bank rows, ids id_base .. id_base+N-1
 * queries [B][d]  stored-type-rounded queries
 * out_ids/out_sims [B][k1]: the min(k1,N) best by (sim desc, id asc); unused slots: id -1, sim -inf.
 * Every similarity is computed and all N pairs are fully sorted.  threads<=1: serial.
 */
int orc_recall(const float* store, int64_t N, int d, int32_t id_base,
               const float* queries, int B, int k1,
               int32_t* out_ids, double* out_sims, int threads) {
    if (N < 0 || d <= 0 || B < 0 || k1 < 1) return 1;
    double* invn = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    if (!invn) return 2;
    for (int64_t n = 0; n < N; ++n) invn[n] = inv_norm(store + n * d, d);
    int failed = 0;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 1 ? threads : 1)
#endif
    for (int b = 0; b < B; ++b) {
        pair_t* all = (pair_t*)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
        if (!all) { failed = 1; continue; }
        const float* q = queries + (int64_t)b * d;
        double invq = inv_norm(q, d);
        for (int64_t n = 0; n < N; ++n) {
            const float* e = store + n * d;
            double dot = 0.0;
            for (int i = 0; i < d; ++i) dot += (double)q[i] * (double)e[i];
            all[n].sim = dot * invq * invn[n];
            all[n].id = id_base + (int32_t)n;
        }
        qsort(all, (size_t)N, sizeof(pair_t), pair_cmp);
        for (int j = 0; j < k1; ++j) {
            if (j < N) { out_ids[(int64_t)b * k1 + j] = all[j].id; out_sims[(int64_t)b * k1 + j] = all[j].sim; }
            else       { out_ids[(int64_t)b * k1 + j] = -1;        out_sims[(int64_t)b * k1 + j] = -INFINITY; }
        }
        free(all);
    }
    free(invn);
    return failed ? 2 : 0;
}

/*
 * Typed / masked recall (Sec. 3.2: items of several types share the bank; Sec. 4.3: entries of held-out
 * operators are left out).  tags[n]: type = tag & 0xff (only types 0..31 can be accepted), group =
 * tag >> 8.  Query b accepts entry n iff bit `type` of allow[b] is set and group != exclude[b].
 * The pool is the top-k1 of the accepted entries, by definition: every accepted pair is scored and
 * all of them are sorted.
 */
int orc_recall_masked(const float* store, int64_t N, int d, const uint32_t* tags,
                      const float* queries, int B, const uint32_t* allow, const uint32_t* exclude, int k1,
                      int32_t* out_ids, double* out_sims) {
    if (N < 0 || d <= 0 || B < 0 || k1 < 1) return 1;
    pair_t* acc = (pair_t*)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
    if (!acc) return 2;
    for (int b = 0; b < B; ++b) {
        const float* q = queries + (int64_t)b * d;
        double invq = inv_norm(q, d);
        int64_t m = 0;
        for (int64_t n = 0; n < N; ++n) {
            uint32_t type = tags[n] & 0xffu, group = tags[n] >> 8;
            if (type > 31u || !((allow[b] >> type) & 1u) || group == exclude[b]) continue;
            const float* e = store + n * d;
            double dot = 0.0;
            for (int i = 0; i < d; ++i) dot += (double)q[i] * (double)e[i];
            acc[m].sim = dot * invq * inv_norm(e, d);
            acc[m].id = (int32_t)n;
            ++m;
        }
        qsort(acc, (size_t)m, sizeof(pair_t), pair_cmp);
        for (int j = 0; j < k1; ++j) {
            if (j < m) { out_ids[(int64_t)b * k1 + j] = acc[j].id; out_sims[(int64_t)b * k1 + j] = acc[j].sim; }
            else       { out_ids[(int64_t)b * k1 + j] = -1;        out_sims[(int64_t)b * k1 + j] = -INFINITY; }
        }
    }
    free(acc);
    return 0;
}

/* Similarities of one query against a given list of ids (used to judge near-ties and to re-rank a
 * candidate set chosen by someone else). */
int orc_sims_of(const float* store, int64_t N, int d, const float* query,
                const int32_t* ids, int count, double* out_sims) {
    double invq = inv_norm(query, d);
    for (int j = 0; j < count; ++j) {
        if (ids[j] < 0 || ids[j] >= N) { out_sims[j] = -INFINITY; continue; }
        const float* e = store + (int64_t)ids[j] * d;
        double dot = 0.0;
        for (int i = 0; i < d; ++i) dot += (double)query[i] * (double)e[i];
        out_sims[j] = dot * invq * inv_norm(e, d);
    }
    return 0;
}

/* ---------- step 2: value filter (re-rank the pool, keep the final items) ---------- */

static void zscores(const double* x, int k, double* z) {
    double mean = 0.0;
    for (int i = 0; i < k; ++i) mean += x[i];
    mean /= (double)k;
    double var = 0.0;
    for (int i = 0; i < k; ++i) var += (x[i] - mean) * (x[i] - mean);
    var /= (double)k;                       /* population variance, as the paper's own running sigma */
    double denom = sqrt(var) + 1e-6;
    for (int i = 0; i < k; ++i) z[i] = (x[i] - mean) / denom;
}

/*
 * One query.  cand_ids/cand_sims: the pool (count entries, ids >= 0).  qtable: the stage's Q values
 * indexed by id.  Writes min(k2,count) results sorted by (score desc, id asc); pads with -1 / -inf.
 * out_scores_f32 may be NULL; out_scores_f64 may be NULL.
 */
int orc_rerank(const int32_t* cand_ids, const double* cand_sims, int count,
               const float* qtable, double lam, int k2,
               int32_t* out_ids, float* out_scores_f32, double* out_scores_f64) {
    if (count < 0 || k2 < 1) return 1;
    double* qv = (double*)malloc(sizeof(double) * (size_t)(count + 1));
    double* zs = (double*)malloc(sizeof(double) * (size_t)(count + 1));
    double* zq = (double*)malloc(sizeof(double) * (size_t)(count + 1));
    pair_t* sc = (pair_t*)malloc(sizeof(pair_t) * (size_t)(count + 1));
    if (count > 0) {
        for (int i = 0; i < count; ++i) qv[i] = (double)qtable[cand_ids[i]];
        zscores(cand_sims, count, zs);
        zscores(qv, count, zq);
        for (int i = 0; i < count; ++i) {
            sc[i].sim = (1.0 - lam) * zs[i] + lam * zq[i];
            sc[i].id = cand_ids[i];
        }
        qsort(sc, (size_t)count, sizeof(pair_t), pair_cmp);
    }
    for (int j = 0; j < k2; ++j) {
        int ok = j < count;
        out_ids[j] = ok ? sc[j].id : -1;
        if (out_scores_f32) out_scores_f32[j] = ok ? (float)sc[j].sim : -INFINITY;
        if (out_scores_f64) out_scores_f64[j] = ok ? sc[j].sim : -INFINITY;
    }
    free(qv); free(zs); free(zq); free(sc);
    return 0;
}

/* ---------- epsilon-greedy selection over the pool (Sec. 3.3, Stage 1: the drafting context is
 * drawn from the pool C(x) by an epsilon-greedy policy; Sec. 4.4 names the same policy) ----------
 *
 * Reading: the k2 slots are filled in order.  For slot j, with probability eps the slot takes a
 * uniformly random member of the pool that is not chosen yet, otherwise the best member not chosen
 * yet (score desc, id asc).  eps = 0 is the plain value filter above.
 * Random numbers: Philox-4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
 * as easy as 1, 2, 3", SC'11), key = the 64-bit seed, counter = (step low, step high, query, slot).
 * Word 0 decides exploration: explore iff word0 < floor(eps * 2^32) (compared as 64-bit integers, so
 * eps = 1 always explores).  Word 1 picks the member: index floor(word1 * remaining / 2^32) into the
 * not-yet-chosen members in greedy order.  Integer decisions only, so both sides agree exactly.
 */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;     /* multipliers M0, M1 of the 4x32 variant */
        uint64_t p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;                                      /* Weyl increments of the key */
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* As orc_rerank, with epsilon-greedy slot filling.  explored (may be NULL) gets 1 for slots filled
 * by the random branch.  query_index is the query's row in its batch (part of the counter). */
int orc_rerank_eps(const int32_t* cand_ids, const double* cand_sims, int count,
                   const float* qtable, double lam, int k2, float eps, uint64_t seed, uint64_t step,
                   uint32_t query_index, int32_t* out_ids, float* out_scores_f32, double* out_scores_f64,
                   unsigned char* explored) {
    if (count < 0 || k2 < 1 || !(eps >= 0.0f && eps <= 1.0f)) return 1;
    int32_t* ord_ids = (int32_t*)malloc(sizeof(int32_t) * (size_t)(count + 1));
    double* ord_sc = (double*)malloc(sizeof(double) * (size_t)(count + 1));
    unsigned char* taken = (unsigned char*)calloc((size_t)(count + 1), 1);
    /* greedy order of the whole pool */
    int rc = orc_rerank(cand_ids, cand_sims, count, qtable, lam, count > 0 ? count : 1, ord_ids, NULL, ord_sc);
    if (rc) { free(ord_ids); free(ord_sc); free(taken); return rc; }
    const uint64_t thr = (uint64_t)((double)eps * 4294967296.0);
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (int j = 0; j < k2; ++j) {
        int remaining = count - j;
        if (remaining <= 0) {
            out_ids[j] = -1;
            if (out_scores_f32) out_scores_f32[j] = -INFINITY;
            if (out_scores_f64) out_scores_f64[j] = -INFINITY;
            if (explored) explored[j] = 0;
            continue;
        }
        const uint32_t ctr[4] = {(uint32_t)step, (uint32_t)(step >> 32), query_index, (uint32_t)j};
        uint32_t rnd[4];
        orc_philox4x32_10(ctr, key, rnd);
        int explore = (uint64_t)rnd[0] < thr;
        int want = explore ? (int)(((uint64_t)rnd[1] * (uint64_t)remaining) >> 32) : 0;   /* index among the free ones */
        int pos = -1;
        for (int i = 0, seen = 0; i < count; ++i) {
            if (taken[i]) continue;
            if (seen == want) { pos = i; break; }
            ++seen;
        }
        taken[pos] = 1;
        out_ids[j] = ord_ids[pos];
        if (out_scores_f32) out_scores_f32[j] = (float)ord_sc[pos];
        if (out_scores_f64) out_scores_f64[j] = ord_sc[pos];
        if (explored) explored[j] = (unsigned char)explore;
    }
    free(ord_ids); free(ord_sc); free(taken);
    return 0;
}

/* ---------- start-point selection (Sec. 3.4) ---------- */

/* One start point out of a task's set P(x), by the refining stage's values (or any stage's table):
 * the member with the largest Q, the lower id among equals (a NaN value counts as -inf); with
 * probability eps instead a uniformly random position of the set (epsilon-greedy, the policy
 * Sec. 4.4 states for start points as for contexts).  ids: the set in the caller's order, n of them;
 * ids outside [0, N) are not members (their number is returned).  The draw is Philox-4x32-10 with
 * key = seed and counter = (step low, step high, set_index, 0xffffffff): word 0 decides (explore iff
 * word0 < floor(eps * 2^32)), word 1 picks position floor(word1 * members / 2^32) among the members
 * in array order.  An empty set gives id -1, value 0, explored 0. */
int64_t orc_select_by_q(const int32_t* ids, int64_t n, const float* qtable, int64_t N, float eps,
                        uint64_t seed, uint64_t step, uint32_t set_index,
                        int32_t* out_id, float* out_q, unsigned char* explored) {
    int64_t members = 0, skipped = 0;
    int32_t best = -1;
    double best_q = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        int32_t id = ids[i];
        if (id < 0 || id >= N) { ++skipped; continue; }
        double q = (double)qtable[id];
        if (q != q) q = -INFINITY;
        if (members == 0 || q > best_q || (q == best_q && id < best)) { best = id; best_q = q; }
        ++members;
    }
    *out_id = -1; *out_q = 0.0f;
    if (explored) *explored = 0;
    if (members == 0) return skipped;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    const uint32_t ctr[4] = {(uint32_t)step, (uint32_t)(step >> 32), set_index, 0xffffffffu};
    uint32_t rnd[4];
    orc_philox4x32_10(ctr, key, rnd);
    const uint64_t thr = (uint64_t)((double)eps * 4294967296.0);
    if ((uint64_t)rnd[0] < thr) {
        int64_t want = (int64_t)(((uint64_t)rnd[1] * (uint64_t)members) >> 32), seen = 0;
        for (int64_t i = 0; i < n; ++i) {
            int32_t id = ids[i];
            if (id < 0 || id >= N) continue;
            if (seen == want) { best = id; break; }
            ++seen;
        }
        if (explored) *explored = 1;
    }
    *out_id = best;
    *out_q = qtable[best];
    return skipped;
}

/* ---------- step 3: unified value update ---------- */

/* Reference: fp64 state seeded from the fp32 table, rounded back to fp32 once at the end.
 * Ids outside [0,N) are skipped; returns how many were skipped. */
int64_t orc_update_q64(float* qtable, int64_t N, const int32_t* ids, const float* rewards,
                       int64_t M, double alpha) {
    double* state = (double*)malloc(sizeof(double) * (size_t)(N > 0 ? N : 1));
    unsigned char* touched = (unsigned char*)calloc((size_t)(N > 0 ? N : 1), 1);
    int64_t skipped = 0;
    for (int64_t n = 0; n < N; ++n) state[n] = (double)qtable[n];
    for (int64_t j = 0; j < M; ++j) {
        int32_t id = ids[j];
        if (id < 0 || id >= N) { ++skipped; continue; }
        state[id] = state[id] + alpha * ((double)rewards[j] - state[id]);
        touched[id] = 1;
    }
    for (int64_t n = 0; n < N; ++n) if (touched[n]) qtable[n] = (float)state[n];
    free(state); free(touched);
    return skipped;
}

/* Same recurrence carried in fp32, one rounding per operation, no fused multiply-add: the value a
 * sequential single-precision implementation reaches bit for bit. */
int64_t orc_update_q32(float* qtable, int64_t N, const int32_t* ids, const float* rewards,
                       int64_t M, float alpha) {
    int64_t skipped = 0;
    for (int64_t j = 0; j < M; ++j) {
        int32_t id = ids[j];
        if (id < 0 || id >= N) { ++skipped; continue; }
        volatile float diff = rewards[j] - qtable[id];
        volatile float step = alpha * diff;
        qtable[id] = qtable[id] + step;
    }
    return skipped;
}

/* ---------- rewards of the two stages and their online normalisation ----------
 *
 * Stage 1 (Sec. 3.3): +1 for a feasible candidate, -1 otherwise.
 * Stage 2 (Sec. 3.4): -1 if infeasible, else tanh(log b - log l) with b the best latency so far and l
 * the measured latency (App. A writes it tanh(log rho) with rho = b / l the speed-up ratio).
 * Normalisation (Sec. 3.4 "PopArt-style", App. A "Stability of Online Normalization"): sample t is
 * mapped to (r_t - mu_{t-1}) / max(sigma_{t-1}, sigma_min), clipped to [-clip, clip] if clip > 0,
 * where mu and sigma are the running mean and POPULATION deviation (1/t form) of all raw rewards
 * seen before it.  Reading: the statistics cover every raw reward of the stage, the -1 of infeasible
 * samples included; before the first sample mu = 0 and sigma = 0 (so the floor applies).
 * state = {count, sum, sum of squares} carries the statistics across calls; fp64 throughout.
 */
int orc_shape_rewards(int stage, const unsigned char* feasible, const float* latency, const float* best_latency,
                      int64_t M, int normalise, double sigma_min, double clip, double state[3], float* out) {
    if ((stage != 0 && stage != 1) || M < 0 || (normalise && !(sigma_min > 0.0))) return 1;
    for (int64_t j = 0; j < M; ++j) {
        double raw;
        if (!feasible[j]) raw = -1.0;
        else if (stage == 0) raw = 1.0;
        else raw = tanh(log((double)best_latency[j]) - log((double)latency[j]));
        double r = raw;
        if (normalise) {
            double n = state[0];
            double mu = n > 0.0 ? state[1] / n : 0.0;
            double var = n > 0.0 ? state[2] / n - mu * mu : 0.0;
            double sigma = var > 0.0 ? sqrt(var) : 0.0;
            double denom = sigma > sigma_min ? sigma : sigma_min;
            r = (raw - mu) / denom;
            if (clip > 0.0) r = r > clip ? clip : (r < -clip ? -clip : r);
            state[0] = n + 1.0;
            state[1] += raw;
            state[2] += raw * raw;
        }
        out[j] = (float)r;
    }
    return 0;
}

int orc_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
