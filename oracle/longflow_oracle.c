/*
 * LongFlow decode-step ORACLE  --  test infrastructure, not product code.
 *
 * A plain, slow, double-precision CPU statement of what one LongFlow decode
 * step computes over a fixed-budget static KV cache.  Only the tests, the
 * smoke check and the benchmark's cpu_baseline leg may call it; the GPU
 * library shares no code, header, table or helper with this file.
 *
 * What it computes, per (batch b, KV head g) unit and per decode step t
 * (ordering: Fig. 2 left -- the new K/V first covers the slot chosen by the
 * previous step, then the cache and the query go through attention):
 *
 *   1. insert    K[slot] <- k_t, V[slot] <- v_t, slot = pending
 *                (pending = count while the cache is still filling)
 *   2. logits    s_h^i = q_h . k^i / sqrt(d_k)              (eq. 1, eq. 4)
 *   3. weights   alpha_h^i = exp(s_h^i) / sum_j exp(s_h^j)  (eq. 1, eq. 4)
 *   4. output    o_h = sum_i alpha_h^i v^i                  (eq. 1)
 *   5. score     LongFlowScore(i) = sum_{h in group} alpha_h^i * ||v^i||_1
 *                (eq. 6 per head; the sum over the query heads that share
 *                 the KV head is this build's reading -- the paper omits
 *                 heads, Sec. 2.1)
 *   6. evict     pending <- argmin_i score(i) once the cache is full,
 *                lowest index on exact ties  (Sec. 3.2 last paragraph,
 *                Alg. 1 post-processing); while filling, pending <- count.
 *
 * Valid slots are a prefix [0, count) by default.  With an explicit mask
 * (the vector M of Alg. 1: masked logits are -inf, so a masked slot has
 * weight and score 0) any subset of slots may be valid, per unit; steps 2-5
 * then run over the valid slots only, and step 6 hands out the lowest
 * invalid slot while there is one (the same "fill before evicting" reading
 * as the prefix case), else the argmin.
 *
 * Comparison rule (the unfused baseline the paper measures its kernel against:
 * in Fig. 1 both sides drop one token per attention call;
 * Sec. 4.1 describes H2O as ranking tokens by accumulated attention scores,
 * Sec. 2.2 as keeping those scores as auxiliary per-token metadata).  With
 * rule 1 the importance of a slot is the attention weight it has received,
 * summed over the query heads of the group and over every step since the
 * token in it was inserted:
 *   5'. acc(i) <- acc(i) + sum_{h in group} alpha_h^i   (acc(slot) <- 0 at insert)
 *   6'. pending <- argmin_i acc(i) once the cache is full.
 * Steps 1-4 are unchanged.  Prefilled rows start at acc = 0 (no prompt
 * attention is defined on this path).  Rule 1 takes no explicit mask.
 *
 * Prompt compression (lfo_compress_prompt): a prompt longer than the budget is
 * cut to the budget once, before decoding, by the observation-window voting of
 * SnapKV, which the paper names for this (Sec. 4.1) without restating it; the
 * reading taken is written out at the function.  The paper prints nothing this
 * step could be checked against: "parity unpinned" by the paper; the function is
 * pinned to the reading (library softmax per window query, numpy convolution for
 * the pooling, a stable sort for the selection, a closed form for equal keys).
 *
 * The method reaches these plain definitions exactly (the fused kernel of
 * Alg. 1 is only a faster route), so the oracle IS the definitions written
 * out.  Max-subtraction inside the softmax is the textbook, exact-arithmetic
 * equivalent of the max-free form in Alg. 1 and keeps exp() in range.
 *
 * Pins (tests, CPU only): naive softmax attention via a library routine,
 * sum(alpha)=1, eq. 6 at group size 1, closed-form argmin cases, the exact
 * leave-one-out identity and bound of App. A.1, invariance of the definitions
 * under Alg. 1's route (any partition into pieces, exponentials without a
 * maximum, normalisation deferred to the end), brute-force argmin, slot-permutation equivariance, and the fill /
 * one-row-changes-per-step invariants of the static cache (Sec. 3.4).
 * The GQA head-sum (step 5 at group size > 1) has no value in the paper to
 * pin it to: "parity unpinned" beyond its reduction to eq. 6 at G = 1.
 *
 * Layouts: every array is dense row-major double.
 *   q [B][Hq][D]   k_new, v_new [B][Hkv][D]   out [B][Hq][D]
 *   cache K, V [B][Hkv][N][D]   scores [B][Hkv][N]   evict_idx [B][Hkv]
 * Query head h reads KV head h / (Hq/Hkv).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define LFO_API __attribute__((visibility("default")))

/* ------------------------------------------------------------------ */
/* Pure per-unit mathematics                                           */
/* ------------------------------------------------------------------ */

/*
 * Attention + LongFlowScore for one KV head and its G query heads over the
 * n valid rows of K, V (each [n][D]).
 *   out   [G][D]   eq. 1
 *   alpha [G][n]   attention weights (may be NULL)
 *   score [n]      sum_h alpha_h^i * sum_l |v^i_l|      eq. 6, summed over h
 */
LFO_API void lfo_attend_unit(int n, int D, int G, const double *q,
                             const double *K, const double *V, double *out,
                             double *alpha, double *score)
{
    double *a = (double *)malloc(sizeof(double) * (size_t)n);
    for (int i = 0; i < n; ++i) score[i] = 0.0;
    for (int h = 0; h < G; ++h) {
        const double *qh = q + (size_t)h * D;
        /* s^i = q . k^i / sqrt(d_k) */
        double smax = -INFINITY;
        for (int i = 0; i < n; ++i) {
            double dot = 0.0;
            for (int l = 0; l < D; ++l) dot += qh[l] * K[(size_t)i * D + l];
            a[i] = dot / sqrt((double)D);
            if (a[i] > smax) smax = a[i];
        }
        /* alpha^i = exp(s^i) / Z, Z = sum_j exp(s^j) */
        double Z = 0.0;
        for (int i = 0; i < n; ++i) {
            a[i] = exp(a[i] - smax);
            Z += a[i];
        }
        for (int i = 0; i < n; ++i) a[i] /= Z;
        /* o = sum_i alpha^i v^i */
        for (int l = 0; l < D; ++l) out[(size_t)h * D + l] = 0.0;
        for (int i = 0; i < n; ++i)
            for (int l = 0; l < D; ++l)
                out[(size_t)h * D + l] += a[i] * V[(size_t)i * D + l];
        /* group score accumulates alpha over the heads sharing this KV head */
        for (int i = 0; i < n; ++i) score[i] += a[i];
        if (alpha) memcpy(alpha + (size_t)h * n, a, sizeof(double) * (size_t)n);
    }
    /* LongFlowScore = alpha * ||v||_1 */
    for (int i = 0; i < n; ++i) {
        double l1 = 0.0;
        for (int l = 0; l < D; ++l) l1 += fabs(V[(size_t)i * D + l]);
        score[i] *= l1;
    }
    free(a);
}

/* argmin with lowest index on exact ties; n >= 1 */
LFO_API int lfo_argmin(int n, const double *x)
{
    int best = 0;
    for (int i = 1; i < n; ++i)
        if (x[i] < x[best]) best = i;
    return best;
}

/* ------------------------------------------------------------------ */
/* Static cache state (Sec. 3.4 "Static Memory and Consistent Workload") */
/* ------------------------------------------------------------------ */

typedef struct lfo_cache {
    int B, Hq, Hkv, D, N, G;
    int count;        /* valid slots = min(tokens seen, N); shared by all units */
    double *K, *V;    /* [B][Hkv][N][D] */
    double *score;    /* [B][Hkv][N], last step; 0 for invalid slots */
    int32_t *pending; /* [B][Hkv] slot the next token's K/V will cover; -1 = none */
    uint8_t *mask;    /* NULL: valid slots are the prefix [0, count); else [B][Hkv][N], 1 = valid */
    int rule;         /* 0: LongFlowScore of the last step (eq. 6); 1: accumulated attention weights */
    double *acc;      /* rule 1: [B][Hkv][N] attention weight received since insertion */
} lfo_cache;

LFO_API lfo_cache *lfo_cache_create(int B, int Hq, int Hkv, int D, int N)
{
    if (B < 1 || Hq < 1 || Hkv < 1 || D < 1 || N < 1 || Hq % Hkv) return NULL;
    lfo_cache *c = (lfo_cache *)calloc(1, sizeof(*c));
    c->B = B; c->Hq = Hq; c->Hkv = Hkv; c->D = D; c->N = N; c->G = Hq / Hkv;
    size_t units = (size_t)B * Hkv;
    c->K = (double *)malloc(sizeof(double) * units * N * D);
    c->V = (double *)malloc(sizeof(double) * units * N * D);
    /* empty slots hold NaN so that any read of them poisons the result */
    for (size_t i = 0; i < units * N * D; ++i) c->K[i] = c->V[i] = NAN;
    c->score = (double *)calloc(units * N, sizeof(double));
    c->pending = (int32_t *)malloc(sizeof(int32_t) * units);
    for (size_t u = 0; u < units; ++u) c->pending[u] = 0;
    c->count = 0;
    return c;
}

LFO_API void lfo_cache_destroy(lfo_cache *c)
{
    if (!c) return;
    free(c->K); free(c->V); free(c->score); free(c->pending); free(c->mask); free(c->acc); free(c);
}

/*
 * Importance rule: 0 = LongFlowScore (eq. 6), 1 = accumulated attention weights
 * (header, steps 5' and 6').  Choosing rule 1 clears the accumulators.
 */
LFO_API int lfo_cache_set_rule(lfo_cache *c, int rule)
{
    if (rule != 0 && rule != 1) return 1;
    if (rule == 1 && c->mask) return 3;
    c->rule = rule;
    if (rule == 1) {
        size_t n = (size_t)c->B * c->Hkv * c->N;
        if (!c->acc) c->acc = (double *)malloc(sizeof(double) * n);
        for (size_t i = 0; i < n; ++i) c->acc[i] = 0.0;
    }
    return 0;
}

/*
 * Prefill: rows [0, n_init) of every unit come from k_init, v_init
 * ([B][Hkv][n_init][D]).  A cache that is not yet full continues to fill at
 * slot n_init; a cache born full has no pending slot until one is set.
 */
LFO_API int lfo_cache_init(lfo_cache *c, const double *k_init,
                           const double *v_init, int n_init)
{
    if (n_init < 0 || n_init > c->N) return 1;
    size_t units = (size_t)c->B * c->Hkv;
    for (size_t u = 0; u < units; ++u) {
        if (n_init) {
            memcpy(c->K + u * c->N * c->D, k_init + u * n_init * c->D,
                   sizeof(double) * (size_t)n_init * c->D);
            memcpy(c->V + u * c->N * c->D, v_init + u * n_init * c->D,
                   sizeof(double) * (size_t)n_init * c->D);
        }
        c->pending[u] = (n_init < c->N) ? n_init : -1;
    }
    c->count = n_init;
    return 0;
}

/*
 * Explicit validity mask (Alg. 1's M), [B][Hkv][N], 1 = valid.  From here on
 * the cache is in mask mode: every step looks at all N slots of a unit.  A
 * unit with an invalid slot gets its lowest one as pending slot; a unit
 * without keeps the pending slot it has.
 */
LFO_API int lfo_cache_set_mask(lfo_cache *c, const uint8_t *mask)
{
    size_t units = (size_t)c->B * c->Hkv;
    if (c->rule == 1) return 3;
    if (!c->mask) c->mask = (uint8_t *)malloc(units * c->N);
    for (size_t i = 0; i < units * c->N; ++i) c->mask[i] = mask[i] ? 1 : 0;
    for (size_t u = 0; u < units; ++u)
        for (int i = 0; i < c->N; ++i)
            if (!c->mask[u * c->N + i]) { c->pending[u] = i; break; }
    c->count = c->N;
    return 0;
}

LFO_API int lfo_cache_get_mask(const lfo_cache *c, uint8_t *mask)
{
    size_t units = (size_t)c->B * c->Hkv;
    for (size_t u = 0; u < units; ++u)
        for (int i = 0; i < c->N; ++i)
            mask[u * c->N + i] = c->mask ? c->mask[u * c->N + i] : (uint8_t)(i < c->count);
    return 0;
}

/*
 * Batch eviction, the "compress every k steps" regime the paper contrasts
 * its per-step eviction with (Sec. 4.4): drop the k valid slots with the
 * lowest LongFlowScore of the last step (eq. 6; lowest index first among
 * equal scores) at once.  They become holes of an explicit mask, which the
 * next k tokens fill lowest-first.  evicted [B][Hkv][k] receives the slots in
 * the order chosen (-1 once a unit has no valid slot left).  k = 1 drops the
 * slot the last step chose anyway.
 */
LFO_API int lfo_cache_evict_lowest(lfo_cache *c, int k, int32_t *evicted)
{
    size_t units = (size_t)c->B * c->Hkv;
    const int N = c->N;
    if (k < 1 || k >= N) return 1;
    if (c->rule == 1) return 3;
    if (!c->mask) { /* the prefix becomes an explicit mask */
        c->mask = (uint8_t *)malloc(units * N);
        for (size_t u = 0; u < units; ++u)
            for (int i = 0; i < N; ++i) c->mask[u * N + i] = (uint8_t)(i < c->count);
    }
    for (size_t u = 0; u < units; ++u) {
        uint8_t *m = c->mask + u * N;
        const double *sc = c->score + u * N;
        for (int j = 0; j < k; ++j) {
            int best = -1;
            for (int i = 0; i < N; ++i)
                if (m[i] && (best < 0 || sc[i] < sc[best])) best = i;
            if (best >= 0) m[best] = 0;
            if (evicted) evicted[u * k + j] = best;
        }
        for (int i = 0; i < N; ++i)
            if (!m[i]) { c->pending[u] = i; break; }
    }
    c->count = N;
    return 0;
}

/* one unit's step in mask mode: steps 1-6 over an arbitrary valid set */
static void step_masked_unit(lfo_cache *c, int u, const double *q, const double *k_new,
                             const double *v_new, double *out, int32_t *evict_idx)
{
    const int D = c->D, N = c->N, G = c->G;
    double *Ku = c->K + (size_t)u * N * D, *Vu = c->V + (size_t)u * N * D;
    uint8_t *m = c->mask + (size_t)u * N;
    double *sc = c->score + (size_t)u * N;
    /* 1. insert; the slot becomes valid */
    const int slot = c->pending[u];
    memcpy(Ku + (size_t)slot * D, k_new + (size_t)u * D, sizeof(double) * D);
    memcpy(Vu + (size_t)slot * D, v_new + (size_t)u * D, sizeof(double) * D);
    m[slot] = 1;
    /* 2-5. attention over the valid rows, gathered side by side */
    int nv = 0;
    for (int i = 0; i < N; ++i) nv += m[i];
    int *idx = (int *)malloc(sizeof(int) * (size_t)nv);
    double *Kg = (double *)malloc(sizeof(double) * (size_t)nv * D);
    double *Vg = (double *)malloc(sizeof(double) * (size_t)nv * D);
    double *sg = (double *)malloc(sizeof(double) * (size_t)nv);
    for (int i = 0, j = 0; i < N; ++i)
        if (m[i]) {
            idx[j] = i;
            memcpy(Kg + (size_t)j * D, Ku + (size_t)i * D, sizeof(double) * D);
            memcpy(Vg + (size_t)j * D, Vu + (size_t)i * D, sizeof(double) * D);
            ++j;
        }
    lfo_attend_unit(nv, D, G, q + (size_t)u * G * D, Kg, Vg, out + (size_t)u * G * D, NULL, sg);
    for (int i = 0; i < N; ++i) sc[i] = 0.0;
    for (int j = 0; j < nv; ++j) sc[idx[j]] = sg[j];
    /* 6. fill the lowest hole if there is one, else evict the minimum score */
    int next = -1;
    for (int i = 0; i < N && next < 0; ++i)
        if (!m[i]) next = i;
    if (next < 0) next = lfo_argmin(N, sc);
    c->pending[u] = next;
    if (evict_idx) evict_idx[u] = next;
    free(idx); free(Kg); free(Vg); free(sg);
}

/*
 * One decode step for every unit (steps 1-6 of the header).
 * Returns 0, or 2 if the cache is full and some unit has no pending slot.
 */
LFO_API int lfo_cache_step(lfo_cache *c, const double *q, const double *k_new,
                           const double *v_new, double *out, int32_t *evict_idx)
{
    const int D = c->D, N = c->N, G = c->G;
    const int units = c->B * c->Hkv;
    for (int u = 0; u < units; ++u)
        if (c->pending[u] < 0 || c->pending[u] >= N) return 2;
    if (c->mask) {
#pragma omp parallel for schedule(dynamic, 1)
        for (int u = 0; u < units; ++u) step_masked_unit(c, u, q, k_new, v_new, out, evict_idx);
        return 0;
    }
    const int n = (c->count < N) ? c->count + 1 : N;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < units; ++u) {
        double *Ku = c->K + (size_t)u * N * D, *Vu = c->V + (size_t)u * N * D;
        /* 1. the new token covers the slot selected by the previous step */
        int slot = c->pending[u];
        memcpy(Ku + (size_t)slot * D, k_new + (size_t)u * D, sizeof(double) * D);
        memcpy(Vu + (size_t)slot * D, v_new + (size_t)u * D, sizeof(double) * D);
        /* 2-5. attention and scores over the n valid rows (a prefix) */
        double *sc = c->score + (size_t)u * N;
        if (c->rule == 1) {
            /* 5'. the slot's history starts over; every valid slot then adds the weight
             * this step's G query heads gave it, and that running sum is its score */
            double *acc = c->acc + (size_t)u * N;
            double *alpha = (double *)malloc(sizeof(double) * (size_t)G * n);
            acc[slot] = 0.0;
            lfo_attend_unit(n, D, G, q + (size_t)u * G * D, Ku, Vu,
                            out + (size_t)u * G * D, alpha, sc);
            for (int i = 0; i < n; ++i) {
                for (int h = 0; h < G; ++h) acc[i] += alpha[(size_t)h * n + i];
                sc[i] = acc[i];
            }
            free(alpha);
        } else {
            lfo_attend_unit(n, D, G, q + (size_t)u * G * D, Ku, Vu,
                            out + (size_t)u * G * D, NULL, sc);
        }
        for (int i = n; i < N; ++i) sc[i] = 0.0;
        /* 6. next slot: keep filling, else evict the minimum score */
        c->pending[u] = (n < N) ? n : lfo_argmin(N, sc);
        if (evict_idx) evict_idx[u] = c->pending[u];
    }
    c->count = n;
    return 0;
}

/*
 * The next T tokens in one call.  By definition T consecutive decode steps:
 * while the cache has room, token t's query attends to the rows present after
 * its own insert, i.e. causally (Sec. 2.1: prefill caches K, V; decoding
 * appends one token's K, V and attends over all of them); once it is full every
 * further token evicts as usual (Sec. 3.2) -- which is also how a prompt longer
 * than the budget is taken in under the method's own rule (the paper hands
 * that case to SnapKV, which it does not define: this build's reading).
 * q [T][B][Hq][D], k_new, v_new [T][B][Hkv][D], out [T][B][Hq][D];
 * evict_idx [B][Hkv] is the last step's.
 */
LFO_API int lfo_cache_fill(lfo_cache *c, int T, const double *q, const double *k_new,
                           const double *v_new, double *out, int32_t *evict_idx)
{
    if (T < 1) return 1;
    const size_t nq = (size_t)c->B * c->Hq * c->D, nk = (size_t)c->B * c->Hkv * c->D;
    for (int t = 0; t < T; ++t) {
        int rc = lfo_cache_step(c, q + t * nq, k_new + t * nk, v_new + t * nk, out + t * nq, evict_idx);
        if (rc) return rc;
    }
    return 0;
}

LFO_API int lfo_cache_count(const lfo_cache *c) { return c->count; }

LFO_API void lfo_cache_scores(const lfo_cache *c, double *scores)
{
    memcpy(scores, c->score, sizeof(double) * (size_t)c->B * c->Hkv * c->N);
}

LFO_API void lfo_cache_get_pending(const lfo_cache *c, int32_t *slots)
{
    memcpy(slots, c->pending, sizeof(int32_t) * (size_t)c->B * c->Hkv);
}

/* steering hook: after a reported near-tie the harness aligns the oracle's
 * next slot with the other implementation so later steps stay comparable */
LFO_API int lfo_cache_set_pending(lfo_cache *c, const int32_t *slots)
{
    size_t units = (size_t)c->B * c->Hkv;
    for (size_t u = 0; u < units; ++u) {
        if (slots[u] < 0 || slots[u] >= c->N) return 1;
        /* while filling, valid rows stay a prefix: only slot == count is legal */
        if (!c->mask && c->count < c->N && slots[u] != c->count) return 1;
    }
    memcpy(c->pending, slots, sizeof(int32_t) * units);
    return 0;
}

LFO_API void lfo_cache_get_kv(const lfo_cache *c, double *K, double *V)
{
    size_t n = (size_t)c->B * c->Hkv * c->N * c->D;
    memcpy(K, c->K, sizeof(double) * n);
    memcpy(V, c->V, sizeof(double) * n);
}

/* ------------------------------------------------------------------ */
/* A prompt longer than the budget (Sec. 4.1, implementation details)   */
/* ------------------------------------------------------------------ */

/*
 * The paper compresses such a prompt to the budget before decoding starts and
 * names the published SnapKV procedure for it without restating it.  The
 * reading taken, with that procedure's parameters as arguments, for one KV
 * head and its G query heads:
 *   - the last W prompt positions are the observation window; window query j
 *     (prompt position T-W+j) attends causally, i.e. over positions
 *     0 .. T-W+j, with the softmax of eq. 1;
 *   - vote(i) = sum over the W window queries and the G heads of alpha(i),
 *     for the prefix positions i < T-W;
 *   - pooled(i) = (sum of vote over the `pool` positions centred on i, those
 *     outside the prefix counting as 0) / pool   (pool odd; 1 = no pooling);
 *   - kept: the keep-W prefix positions with the largest pooled vote (lowest
 *     position first among equals), in ascending position order, followed by
 *     the W window positions.
 *   q_window [W][G][D], K [T][D]; pooled [T-W] (may be NULL), kept [keep].
 * Returns nonzero if the arguments are out of range (1 <= W <= keep <= T,
 * pool odd and >= 1).
 */
LFO_API int lfo_compress_prompt_unit(int T, int W, int keep, int pool, int D, int G,
                                     const double *q_window, const double *K,
                                     double *pooled_out, int32_t *kept)
{
    if (W < 1 || keep < W || keep > T || pool < 1 || (pool & 1) == 0) return 1;
    const int P = T - W; /* prefix positions */
    double *vote = (double *)calloc((size_t)(P > 0 ? P : 1), sizeof(double));
    double *a = (double *)malloc(sizeof(double) * (size_t)T);
    for (int j = 0; j < W; ++j) {
        const int n = P + j + 1; /* positions this query sees */
        for (int h = 0; h < G; ++h) {
            const double *qh = q_window + ((size_t)j * G + h) * D;
            double smax = -INFINITY, Z = 0.0;
            for (int i = 0; i < n; ++i) {
                double dot = 0.0;
                for (int l = 0; l < D; ++l) dot += qh[l] * K[(size_t)i * D + l];
                a[i] = dot / sqrt((double)D);
                if (a[i] > smax) smax = a[i];
            }
            for (int i = 0; i < n; ++i) { a[i] = exp(a[i] - smax); Z += a[i]; }
            for (int i = 0; i < P; ++i) vote[i] += a[i] / Z;
        }
    }
    double *pooled = (double *)malloc(sizeof(double) * (size_t)(P > 0 ? P : 1));
    for (int i = 0; i < P; ++i) {
        double sum = 0.0;
        for (int d = -(pool / 2); d <= pool / 2; ++d)
            if (i + d >= 0 && i + d < P) sum += vote[i + d];
        pooled[i] = sum / pool;
    }
    /* the keep-W largest, lowest position first among equals: pick them one by one */
    const int kp = keep - W;
    uint8_t *taken = (uint8_t *)calloc((size_t)(P > 0 ? P : 1), 1);
    for (int r = 0; r < kp; ++r) {
        int best = -1;
        for (int i = 0; i < P; ++i)
            if (!taken[i] && (best < 0 || pooled[i] > pooled[best])) best = i;
        taken[best] = 1;
    }
    int d = 0;
    for (int i = 0; i < P; ++i)
        if (taken[i]) kept[d++] = i;
    for (int j = 0; j < W; ++j) kept[d++] = P + j;
    if (pooled_out) memcpy(pooled_out, pooled, sizeof(double) * (size_t)P);
    free(vote); free(a); free(pooled); free(taken);
    return 0;
}

/* the same for every (batch, KV head) unit: q_window [W][B][Hq][D], K [B][Hkv][T][D],
 * pooled [B][Hkv][T-W] (may be NULL), kept [B][Hkv][keep] */
LFO_API int lfo_compress_prompt(int B, int Hq, int Hkv, int D, int T, int W, int keep, int pool,
                                const double *q_window, const double *K, double *pooled, int32_t *kept)
{
    if (B < 1 || Hkv < 1 || Hq % Hkv) return 1;
    const int G = Hq / Hkv;
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int u = 0; u < B * Hkv; ++u) {
        const int b = u / Hkv, g = u % Hkv;
        double *qw = (double *)malloc(sizeof(double) * (size_t)W * G * D);
        for (int j = 0; j < W; ++j)
            memcpy(qw + (size_t)j * G * D, q_window + (((size_t)j * B + b) * Hq + (size_t)g * G) * D,
                   sizeof(double) * (size_t)G * D);
        if (lfo_compress_prompt_unit(T, W, keep, pool, D, G, qw, K + (size_t)u * T * D,
                                     pooled ? pooled + (size_t)u * (T - W) : NULL, kept + (size_t)u * keep))
            bad = 1;
        free(qw);
    }
    return bad;
}

LFO_API int lfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
