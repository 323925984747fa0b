/*
 * longflow.h -- C ABI of the LongFlow fused decode step for AMD MI355X (gfx950).
 *
 * One call of longflow_decode_step() is one pass of the paper's fused
 * attention + importance + eviction operator (Sec. 3.4 "Fused Attention and
 * Eviction Kernel", Alg. 1, Fig. 2) over a fixed-budget static KV cache
 * (Sec. 3.4 "Static Memory and Consistent Workload"), for every
 * (batch, KV head) pair of one layer:
 *
 *   insert   the new token's K/V covers the slot chosen by the previous call
 *            (Fig. 2 left); while the cache is still filling, the next empty slot
 *   attend   o_h = softmax(q_h K^T / sqrt(d_k)) V over the valid slots, for the
 *            query heads h that share the KV head            (eq. 1, eq. 4)
 *   score    LongFlowScore(i) = sum_h alpha_h^i * ||v^i||_1  (eq. 6; the sum over
 *            the group's query heads is this library's reading, the paper
 *            leaves heads out)
 *   evict    next slot = argmin_i LongFlowScore(i), lowest index on ties
 *            (Sec. 3.2, Alg. 1 post-processing); while filling: = valid count
 *
 * Conventions
 *   - Every pointer marked "device" is HIP device memory on the current device;
 *     the CALLER owns all of it (cache, workspace, inputs, outputs) and the
 *     stream.  The library owns only the small host-side handle and never
 *     allocates or frees device memory.
 *   - All tensors are dense, row-major, innermost dimension head_dim, of the
 *     dtype in lf_config (LF_F32 = IEEE binary32, LF_BF16 = bfloat16 bits),
 *     except where a C type is given.  Query head h reads KV head
 *     h / (q_heads / kv_heads).
 *   - Calls are asynchronous on `hip_stream` (a hipStream_t passed as void*,
 *     NULL = the default stream) and never synchronise with the host.  The
 *     sequences of a cache advance in lock-step: one valid-slot count for all.
 *   - Every function returns an lf_status.  Argument errors are detected on the
 *     host before anything is launched and leave the cache untouched.  The text
 *     of the last error of the calling thread is in longflow_last_error().
 *   - Calls on one handle must be serialised by the caller; different handles
 *     are independent (one handle = one layer's cache).
 *   - A decode step of a full cache is a fixed sequence of kernel launches with fixed
 *     arguments (Sec. 3.4: static memory, consistent workload), so it may be captured
 *     into a HIP graph and replayed.  The capture holds the valid-slot count and the
 *     cache's mode: capture only once the cache is full, and again after
 *     longflow_set_mask or longflow_evict_lowest.
 */
#ifndef LONGFLOW_H
#define LONGFLOW_H

#include <stddef.h>
#include <stdint.h>

#if defined(__GNUC__) || defined(__clang__)
#define LF_API __attribute__((visibility("default")))
#else
#define LF_API
#endif

#ifdef __cplusplus
extern "C" {
#endif

typedef struct longflow_cache longflow_cache_t; /* opaque, host memory, library-owned */

typedef enum {
    LF_OK = 0,
    LF_ERR_INVALID_ARG = 1, /* NULL pointer, size out of range                         */
    LF_ERR_UNSUPPORTED = 2, /* geometry the kernels do not cover                       */
    LF_ERR_WORKSPACE = 3,   /* workspace smaller than longflow_workspace_bytes()       */
    LF_ERR_STATE = 4,       /* call out of order (e.g. full cache without pending slot)*/
    LF_ERR_HIP = 5          /* a HIP runtime call or launch failed                      */
} lf_status;

typedef enum { LF_F32 = 0, LF_BF16 = 1 } lf_dtype;

/* flags */
#define LF_FLAG_ATTENTION_ONLY 1u /* plain decode attention: no insert, score or eviction
                                     (the uncompressed comparison of Sec. 4.4)            */
#define LF_FLAG_FORCE_VALU 2u     /* use the vector-ALU kernel instead of a matrix-core
                                     kernel (for A/B measurement)                          */
#define LF_FLAG_FORCE_SPLIT 4u    /* always split a unit over several workgroups              */
#define LF_FLAG_FORCE_UNIT 8u     /* always one workgroup per unit, one fused launch; needs the
                                     matrix-core path and budget * group <= ~120k            */
#define LF_FLAG_UNFUSED_ACCUM 16u /* comparison path, bf16 / head_dim 128 only: the baseline
                                     the paper measures its kernel against (Fig. 1; Sec. 4.1,
                                     "H2O": accumulated attention scores kept as per-token
                                     metadata, Sec. 2.2).  A slot's importance is the attention
                                     weight it has received, summed over the group's query heads
                                     and over every step since its token was inserted (0 for
                                     prefilled rows); the slot with the least is evicted, lowest
                                     slot among equals.  Computed the unfused way: a plain
                                     attention kernel, then separate kernels that re-derive the
                                     weights from K and add them to a per-slot fp32 buffer.
                                     longflow_decode_step keeps its meaning and arguments
                                     (k_new, v_new 16-byte aligned), longflow_scores returns
                                     the accumulated weights; masks, batch eviction and groups
                                     are LF_ERR_UNSUPPORTED.                                  */

#define LF_FLAG_MAX_FREE 32u      /* bf16 / head_dim 128, fused kernel: the softmax exactly as Alg. 1
                                     prints it (Sec. 3.4, modification 2) -- no running reference,
                                     p = exp(s) in fp32, normalised at the end -- in the evicting step
                                     or, with LF_FLAG_ATTENTION_ONLY, in plain attention.  Same values
                                     while every |s| stays below ~88; non-finite output beyond.  The
                                     eviction decision stays exact (its screening bounds turn one-sided
                                     where a slot's ||v||_1 exp(s) leaves [2^-48, 2^16], which only costs
                                     time).  For A/B measurement against the default, which keeps a
                                     reference.  Such a cache takes no mask, batch eviction or group, and
                                     longflow_fill_steps feeds it token by token.                      */

typedef struct {
    int32_t batch;    /* B   >= 1                                            */
    int32_t q_heads;  /* Hq, a multiple of kv_heads.  Hq/Hkv <= 16 (matrix-core kernels);
                         <= 8 with LF_FLAG_FORCE_VALU (vector-ALU kernel):
                         LF_ERR_UNSUPPORTED beyond */
    int32_t kv_heads; /* Hkv >= 1                                            */
    int32_t head_dim; /* D: 64 or 128                                        */
    int32_t budget;   /* N: slots of the static cache, 1 <= N <= 2^24        */
    int32_t dtype;    /* lf_dtype                                            */
    uint32_t flags;   /* LF_FLAG_*                                           */
} lf_config;

/* Bytes of device workspace a cache with this geometry needs (0 if cfg is invalid). */
LF_API size_t longflow_workspace_bytes(const lf_config *cfg);

/*
 * How longflow_init_cache carves the workspace (host-only query; launches nothing, needs no
 * GPU): the regions in address order, each with its byte offset from the (256-byte aligned)
 * workspace base and the bytes the kernels may index in it.  With regions == NULL only the
 * count is returned in *n_regions.  For bounds checks on the host: regions never overlap and
 * end inside longflow_workspace_bytes(cfg).
 */
typedef struct {
    char name[24];
    uint64_t offset;
    uint64_t bytes;
} lf_region;
LF_API int longflow_workspace_regions(const lf_config *cfg, lf_region *regions, int32_t max_regions,
                                      int32_t *n_regions);

/*
 * Create a cache over caller-owned storage (prefill stage of Sec. 2.1).
 *   k_cache, v_cache  device [B][Hkv][N][D]; mutated in place by later calls.
 *                     Slots >= the valid count are never read.
 *   k_init, v_init    device [B][Hkv][n_init][D] copied into slots [0, n_init);
 *                     may be NULL iff n_init == 0.
 *   n_init            0 <= n_init <= N.  If n_init < N the cache keeps filling
 *                     from slot n_init.  If n_init == N there is no slot for the
 *                     next token until longflow_set_pending() names one.
 *   workspace         device, >= longflow_workspace_bytes(cfg), 256-byte aligned,
 *                     kept alive and untouched by the caller until destroy.
 * On success *out receives the handle.
 */
LF_API int longflow_init_cache(longflow_cache_t **out, const lf_config *cfg,
                        void *k_cache, void *v_cache,
                        const void *k_init, const void *v_init, int32_t n_init,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * One fused decode step (Alg. 1 plus the slot write of Fig. 2 left).
 *   q          device [B][Hq][D]
 *   k_new,v_new device [B][Hkv][D]: the current token's key/value
 *   out        device [B][Hq][D], attention output, rounded to nearest even
 *   evict_idx  device int32 [B][Hkv] or NULL: the slot the NEXT call will
 *              overwrite (= valid count while the cache is filling)
 * With LF_FLAG_ATTENTION_ONLY k_new, v_new and evict_idx are ignored and the
 * cache is not modified.
 */
LF_API int longflow_decode_step(longflow_cache_t *cache, const void *q,
                         const void *k_new, const void *v_new,
                         void *out, int32_t *evict_idx, void *hip_stream);

/*
 * The next T tokens in one call, with the results of T consecutive
 * longflow_decode_step calls -- token t attends to the rows present after its own
 * insert (Sec. 2.1: prefill caches K and V, decoding appends one token's and
 * attends over all).  While a cache is filling nothing is evicted, so the steps
 * depend on each other only through the appended rows: for the tokens that find a
 * free slot, bf16 / head_dim 128 caches write all rows first and take the queries
 * through attention several at a time, reading the cache once per
 * 24 * floor(16 / (Hq/Hkv)) tokens (the fill phase in bulk; there the weights enter the
 * P V product rounded to bf16, as fused attention kernels commonly do, so an attention
 * output can differ from the single step's by one unit in the last place of bf16 -- rows,
 * decision and scores are the same).  Tokens beyond the
 * free slots -- a prompt longer than the budget, which the paper hands to an
 * external method -- evict one slot each under the method's own rule (Sec. 3.2),
 * as ordinary steps issued back to back; so do all tokens of caches without the
 * batched kernel or with an explicit mask in force.
 *   q           device [T][B][Hq][D]
 *   k_new,v_new device [T][B][Hkv][D]
 *   out         device [T][B][Hq][D]
 *   evict_idx   device int32 [B][Hkv] or NULL: as after the last of the T steps
 * All pointers 16-byte aligned.  LF_ERR_INVALID_ARG if T < 1; LF_ERR_STATE for a
 * full cache without a pending slot; LF_ERR_UNSUPPORTED with LF_FLAG_ATTENTION_ONLY
 * or LF_FLAG_UNFUSED_ACCUM.  Those are found before anything is launched.  If a launch
 * itself fails part-way (LF_ERR_HIP) the cache holds the tokens issued up to there and
 * longflow_valid_count says how many rows that is.
 */
LF_API int longflow_fill_steps(longflow_cache_t *cache, int32_t T, const void *q,
                        const void *k_new, const void *v_new,
                        void *out, int32_t *evict_idx, void *hip_stream);

/*
 * A prompt longer than the budget, cut down once before decoding starts.  The paper does this
 * with SnapKV and does not restate it (Sec. 4.1, implementation details); the reading built
 * here, per (batch, KV head) with its Hq/Hkv query heads, T prompt rows, the last W of them the
 * observation window, P = T - W the prefix:
 *   - window query j (prompt row P + j) attends causally, over rows 0 .. P + j, with the softmax
 *     of eq. 1;
 *   - vote(i) = sum over the W window queries and the group's query heads of the attention
 *     weight of prefix row i;
 *   - pooled(i) = (sum of vote over the `pool` rows centred on i, rows outside the prefix
 *     counting as 0) / pool;
 *   - kept: the keep - W prefix rows with the largest pooled vote (lowest row among equals), in
 *     prompt order, then the W window rows; they become slots 0 .. keep - 1 of the cache.
 * Afterwards the cache holds `keep` valid rows and goes on exactly as one created with
 * longflow_init_cache(n_init = keep): it keeps filling if keep < N, and with keep == N needs
 * longflow_set_pending before the first step.
 *   q_window  device [W][B][Hq][D]: the queries of the last W prompt rows
 *   k_prompt, v_prompt  device [B][Hkv][T][D]; read only
 *   keep      W <= keep <= min(T, N);  pool: odd, 1 (no pooling) .. 1023
 *   scratch   device, >= longflow_compress_scratch_bytes(cfg, T, W), 256-byte aligned, free for
 *             reuse once the call's work on hip_stream has run
 *   pooled    device float [B][Hkv][T - W] or NULL: the pooled votes (fp32 arithmetic)
 *   kept      device int32 [B][Hkv][keep] or NULL: the prompt rows now in slots 0 .. keep - 1
 * All pointers 16-byte aligned.  LF_ERR_STATE unless the cache is empty (created with
 * n_init = 0, no step, no mask); LF_ERR_UNSUPPORTED for fp32 or head_dim 64 caches, with
 * LF_FLAG_ATTENTION_ONLY / LF_FLAG_FORCE_VALU / LF_FLAG_UNFUSED_ACCUM, for W * Hq/Hkv > 4096 and
 * for B * Hkv * T >= 2^27.  Errors are found before anything is launched.
 */
LF_API size_t longflow_compress_scratch_bytes(const lf_config *cfg, int32_t T, int32_t W);
LF_API int longflow_compress_prompt(longflow_cache_t *cache, int32_t T, int32_t W, int32_t keep, int32_t pool,
                                    const void *q_window, const void *k_prompt, const void *v_prompt,
                                    void *scratch, size_t scratch_bytes, float *pooled, int32_t *kept,
                                    void *hip_stream);

/*
 * LongFlowScore of every slot as of the most recent decode step (the vector
 * S_final_loss of Alg. 1): device float [B][Hkv][N], 0 for invalid slots.
 * Recomputed on demand from the cache and that step's query; not part of the
 * per-step cost.  LF_ERR_STATE before the first step.
 */
LF_API int longflow_scores(longflow_cache_t *cache, float *scores, void *hip_stream);

/* Name the slot the next call overwrites -- the "slot selected in the previous step" that the
 * current K/V covers in Fig. 2 left, here chosen by the caller (resume from saved state, a cache
 * created full, tests): device int32 [B][Hkv], each in [0, N).  Only legal once the cache is
 * full; while it is filling the next slot is the valid count (Sec. 3.4, static memory). */
LF_API int longflow_set_pending(longflow_cache_t *cache, const int32_t *slots, void *hip_stream);

/*
 * Explicit validity mask, the vector M of Alg. 1: device uint8 [B][Hkv][N], nonzero = the
 * slot holds a token.  Any subset may be valid, separately per (batch, KV head): ragged
 * batches, sequences restarted in place, slots dropped by the caller.  As in Alg. 1 an
 * invalid slot has logit -inf, weight 0 and score 0.  From this call on every step looks
 * at all N slots; the slot handed out for the next token is the lowest invalid one while
 * there is one (nothing is evicted before the holes are used up), else the argmin.
 * Effects, in stream order: the K/V rows of invalid slots are overwritten with zeros; a
 * (batch, KV head) that has an invalid slot gets its lowest one as pending slot, one that
 * has none keeps the pending slot it had (a cache created full still needs
 * longflow_set_pending first).  longflow_valid_count then reports N.  Not available
 * with LF_FLAG_ATTENTION_ONLY (LF_ERR_UNSUPPORTED).  May be called again at any time.
 */
LF_API int longflow_set_mask(longflow_cache_t *cache, const uint8_t *mask, void *hip_stream);

/* Which slots hold a token right now: device uint8 [B][Hkv][N], 1 = valid.  Without an
 * explicit mask that is the prefix [0, valid count).  Together with the K/V buffers and
 * the last evict_idx this is the whole state of a cache (save / resume). */
LF_API int longflow_get_mask(longflow_cache_t *cache, uint8_t *mask, void *hip_stream);

/*
 * Batch eviction: the "compress every k steps" regime that Sec. 4.4 sets against the
 * method's own one-slot-per-step eviction, served from the same score (eq. 6).  Drops the
 * k valid slots of every (batch, KV head) with the lowest LongFlowScore of the most recent
 * decode step (double precision; lowest slot first among equal scores); with k = 1 that is
 * the slot the step itself chose.  The dropped slots, and the unfilled ones of a cache that
 * is still filling, become invalid slots of the explicit mask (see longflow_set_mask: rows
 * zeroed, every later step looks at all N slots), so the next tokens refill them lowest
 * slot first and per-step eviction resumes once they are used up.
 *   k        1 <= k < N; a unit with fewer valid slots loses all of them
 *   scratch  device, >= longflow_evict_scratch_bytes(cfg), 8-byte aligned, free for reuse
 *            once the call's work on hip_stream has run
 *   evicted  device int32 [B][Hkv][k], the dropped slots in the order chosen (-1 where a
 *            unit ran out of valid slots), or NULL
 * LF_ERR_STATE before the first decode step; LF_ERR_UNSUPPORTED with LF_FLAG_ATTENTION_ONLY.
 */
LF_API size_t longflow_evict_scratch_bytes(const lf_config *cfg);
LF_API int longflow_evict_lowest(longflow_cache_t *cache, int32_t k, void *scratch, size_t scratch_bytes,
                                 int32_t *evicted, void *hip_stream);

/*
 * longflow_evict_lowest for callers that cannot allocate device memory or pass a scratch
 * buffer: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments minus the scratch, same kernels, same results; the
 * double-precision scores go to a device array built into the library (8 MiB, held by
 * every GPU the library runs on until the process ends; its address on a GPU is resolved
 * by longflow_init_cache on that GPU).  The call allocates and frees nothing.
 *   limit    batch * kv_heads * budget <= LF_EVICT_STATIC_MAX_SLOTS, else LF_ERR_WORKSPACE
 *            (nothing launched, cache untouched): use longflow_evict_lowest instead
 * All calls on one GPU share the one array: calls whose work overlaps on a GPU (different
 * streams, different caches) race on it and must be serialised by the caller.  Nothing in
 * it needs clearing between calls: each call writes every entry it reads.
 */
#define LF_EVICT_STATIC_MAX_SLOTS (1u << 20)
LF_API int longflow_evict_lowest_static(longflow_cache_t *cache, int32_t k, int32_t *evicted, void *hip_stream);

/* Valid slots = min(tokens seen, N); negative on a NULL handle. */
LF_API int longflow_valid_count(const longflow_cache_t *cache);

/* Frees the host handle only.  LF_ERR_STATE while a group still holds the cache. */
LF_API int longflow_destroy_cache(longflow_cache_t *cache);

/*
 * How a configuration will be executed (host-only query; launches nothing, needs no GPU).
 * The kernels all compute the same step (Alg. 1 with the post-processing of Sec. 3.4); the
 * choice below is about filling the chip, not about the result.
 */
typedef enum {
    LF_PATH_SPLIT_VALU = 0, /* split-K, vector ALU (LF_FLAG_FORCE_VALU)                          */
    LF_PATH_SPLIT_MFMA = 1, /* split-K, matrix cores, bf16 head_dim 128 (codes exceed LDS,
                               LF_FLAG_FORCE_SPLIT)                                              */
    LF_PATH_UNIT_MFMA = 2,  /* fused kernel, 1..8 cooperating workgroups per (batch, KV head)    */
    LF_PATH_SPLIT_MFMA_F32 = 3 /* split-K, matrix cores in fp32 arithmetic (fp32 caches; bf16
                               with head_dim 64)                                                 */
} lf_path;
typedef struct {
    int32_t path;                /* lf_path                                                        */
    int32_t workgroups_per_unit; /* at a full cache                                                 */
    int32_t slots_per_workgroup; /* slot range one workgroup streams                                */
    int32_t launches_per_step;   /* 1, or 2 when a large split-K grid (several workgroups per unit) takes a
                                    separate finish launch */
    int32_t threads_per_workgroup;
    uint32_t lds_bytes;          /* dynamic LDS per workgroup (0 on the split-K paths: static only) */
} lf_plan_info;
LF_API int longflow_plan_info(const lf_config *cfg, lf_plan_info *info);

/*
 * Several caches in one launch.  The method's workload is the same every step (Sec. 3.4:
 * static memory, one fused kernel), so caches that are independent of each other --
 * micro-batches, or the layers of a synthetic benchmark -- can share one grid: the launch
 * and the drain between kernels are paid once per group, and a small cache no longer
 * leaves most of the chip idle.  Each member gets what longflow_decode_step computes for
 * it, from the same kernels.  Where the group serves a (batch, KV head) pair with fewer
 * cooperating workgroups than the cache would use on its own, the partial sums of `out`
 * are merged in another order and may differ from a lone call's in the last bits; the
 * eviction index comes from the same exact re-scoring either way.
 *
 *   longflow_group_workspace_bytes  device bytes a group of n_caches needs (0 if n_caches < 1)
 *   longflow_group_create   caches: host array of n_caches handles with identical lf_config
 *                           and the same valid count; workspace: device, 256-byte aligned,
 *                           owned by the caller, must outlive the group.  Writes a table of
 *                           per-cache pointers into it with small kernels on hip_stream
 *                           (asynchronous like every other call).
 *   longflow_group_decode_step  one decode step of every member.  q/out are device
 *                           [n_caches][B][Hq][D], k_new/v_new [n_caches][B][Hkv][D],
 *                           evict_idx int32 [n_caches][B][Hkv] or NULL; otherwise as
 *                           longflow_decode_step.  Members may also be stepped one by one
 *                           between group steps; LF_ERR_STATE if their counts then differ.
 *   longflow_group_destroy  frees the host handle only.  longflow_destroy_cache refuses
 *                           (LF_ERR_STATE) a cache that is still a member of a live group.
 */
typedef struct longflow_group longflow_group_t;
LF_API size_t longflow_group_workspace_bytes(int32_t n_caches);
LF_API int longflow_group_create(longflow_group_t **group, longflow_cache_t *const *caches, int32_t n_caches,
                                 void *workspace, size_t workspace_bytes, void *hip_stream);
LF_API int longflow_group_decode_step(longflow_group_t *group, const void *q, const void *k_new,
                                      const void *v_new, void *out, int32_t *evict_idx, void *hip_stream);
LF_API int longflow_group_destroy(longflow_group_t *group);

/*
 * Measurement aid (not part of the paper's operator): while profiling is on, every
 * decode step records two HIP events on its stream around its kernel launches (one
 * launch per step, two on the split-K path when its grid is large).
 *   longflow_profile_begin  creates events for up to max_steps steps and switches it on
 *   longflow_profile_end    waits for the recorded events, writes the summed kernel
 *                           duration in milliseconds to *kernel_ms and the number of steps
 *                           recorded to *steps (host pointers), destroys the events and
 *                           switches it off.
 * Steps beyond max_steps run untimed.  Synchronises the host with the stream.
 */
LF_API int longflow_profile_begin(longflow_cache_t *cache, int32_t max_steps);
LF_API int longflow_profile_end(longflow_cache_t *cache, float *kernel_ms, int32_t *steps);

/* Text of the calling thread's last error ("" if none). Never NULL. */
LF_API const char *longflow_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LONGFLOW_H */
