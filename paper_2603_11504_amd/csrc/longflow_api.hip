// C ABI of the LongFlow decode step: argument checking, workspace carving, launch order.
// All arithmetic lives in the kernels; nothing here touches cache contents on the host.
#include "../../include/longflow.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "lf_host.h"

namespace lf {

static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }


void choose_splits(int units, int N, int *L, int *C)
{
    // Enough workgroups to fill 256 CUs several times over, each streaming a span long
    // enough to amortise its prologue/merge; spans are multiples of 256 slots.
    long c = (2048 + units - 1) / units;
    const long c_span = (N + 2047) / 2048;           // spans no longer than 2048 slots
    if (c < c_span) c = c_span;
    if (c > kMaxSplits) c = kMaxSplits;
    if (c < 1) c = 1;
    long l = (N + c - 1) / c;
    l = (l + 255) / 256 * 256;
    while ((N + l - 1) / l > kMaxSplits) l += 256;
    *L = (int)l;
    *C = (int)((N + l - 1) / l);
}

static int validate(const lf_config *cfg)
{
    if (!cfg) return fail(LF_ERR_INVALID_ARG, "cfg is NULL");
    if (cfg->batch < 1 || cfg->q_heads < 1 || cfg->kv_heads < 1 || cfg->budget < 1 ||
        cfg->budget > (1 << 24))
        return fail(LF_ERR_INVALID_ARG, "batch/heads/budget out of range");
    if (cfg->dtype != LF_F32 && cfg->dtype != LF_BF16)
        return fail(LF_ERR_INVALID_ARG, "unknown dtype %d", cfg->dtype);
    if (cfg->flags & ~(LF_FLAG_ATTENTION_ONLY | LF_FLAG_FORCE_VALU | LF_FLAG_FORCE_SPLIT | LF_FLAG_FORCE_UNIT |
                       LF_FLAG_UNFUSED_ACCUM | LF_FLAG_MAX_FREE))
        return fail(LF_ERR_INVALID_ARG, "unknown flag bits 0x%x", cfg->flags);
    if (cfg->q_heads % cfg->kv_heads)
        return fail(LF_ERR_UNSUPPORTED, "q_heads %d is not a multiple of kv_heads %d", cfg->q_heads,
                    cfg->kv_heads);
    if (cfg->head_dim != 64 && cfg->head_dim != 128)
        return fail(LF_ERR_UNSUPPORTED, "head_dim %d (supported: 64, 128)", cfg->head_dim);
    const int G = cfg->q_heads / cfg->kv_heads;
    if (G > kMaxGroup) return fail(LF_ERR_UNSUPPORTED, "group size %d > %d", G, kMaxGroup);
    const bool mfma = cfg->dtype == LF_BF16 && cfg->head_dim == 128 && !(cfg->flags & LF_FLAG_FORCE_VALU);
    if ((cfg->flags & LF_FLAG_FORCE_VALU) && G > 8)
        return fail(LF_ERR_UNSUPPORTED, "group size %d > 8 needs a matrix-core kernel (drop FORCE_VALU)", G);
    if ((long long)cfg->batch * cfg->kv_heads > (1ll << 20))
        return fail(LF_ERR_UNSUPPORTED, "batch*kv_heads > 2^20");
    if ((cfg->flags & LF_FLAG_FORCE_SPLIT) && (cfg->flags & LF_FLAG_FORCE_UNIT))
        return fail(LF_ERR_INVALID_ARG, "FORCE_SPLIT and FORCE_UNIT exclude each other");
    if (cfg->flags & LF_FLAG_UNFUSED_ACCUM) {
        if (cfg->flags & (LF_FLAG_ATTENTION_ONLY | LF_FLAG_FORCE_VALU))
            return fail(LF_ERR_INVALID_ARG, "UNFUSED_ACCUM excludes ATTENTION_ONLY and FORCE_VALU");
        if (!mfma) return fail(LF_ERR_UNSUPPORTED, "UNFUSED_ACCUM needs bf16 and head_dim 128");
        if ((long long)cfg->batch * cfg->kv_heads * (cfg->budget + kTile) >= (1ll << 31))
            return fail(LF_ERR_UNSUPPORTED, "UNFUSED_ACCUM: batch*kv_heads*budget >= 2^31");
    }
    if (cfg->flags & LF_FLAG_MAX_FREE) {
        if (cfg->flags & LF_FLAG_UNFUSED_ACCUM) return fail(LF_ERR_INVALID_ARG, "MAX_FREE and UNFUSED_ACCUM exclude each other");
        if (!mfma || (cfg->flags & LF_FLAG_FORCE_SPLIT))
            return fail(LF_ERR_UNSUPPORTED, "MAX_FREE needs bf16, head_dim 128 and the fused matrix-core kernel");
    }
    if (cfg->flags & LF_FLAG_FORCE_UNIT) {
        if (!mfma) return fail(LF_ERR_UNSUPPORTED, "FORCE_UNIT needs bf16, head_dim 128 and the matrix-core kernel");
        if (unit_mfma_lds_bytes(cfg->budget, G, !(cfg->flags & (LF_FLAG_ATTENTION_ONLY | LF_FLAG_UNFUSED_ACCUM)), 1) > kUnitLdsLimit)
            return fail(LF_ERR_UNSUPPORTED, "FORCE_UNIT: budget %d x group %d does not fit one workgroup's LDS", cfg->budget, G);
    }
    return LF_OK;
}

static void fill_plan(const lf_config *cfg, Plan *p)
{
    memset(p, 0, sizeof(*p));
    p->B = cfg->batch; p->Hq = cfg->q_heads; p->Hkv = cfg->kv_heads; p->D = cfg->head_dim;
    p->N = cfg->budget; p->G = cfg->q_heads / cfg->kv_heads; p->units = cfg->batch * cfg->kv_heads;
    p->dtype = cfg->dtype; p->flags = cfg->flags;
    // the comparison path runs the plain attention kernels: that is the flag they see
    p->unfused = cfg->flags & LF_FLAG_UNFUSED_ACCUM;
    if (p->unfused) p->flags = (cfg->flags & ~LF_FLAG_UNFUSED_ACCUM) | LF_FLAG_ATTENTION_ONLY;
    p->max_free = cfg->flags & LF_FLAG_MAX_FREE;
    choose_splits(p->units, p->N, &p->L, &p->C);
    p->ntiles = (p->N + kTile - 1) / kTile;
    p->use_mfma = cfg->dtype == LF_BF16 && cfg->head_dim == 128 && !(cfg->flags & LF_FLAG_FORCE_VALU);
    p->use_mfma32 = !p->use_mfma && !(cfg->flags & LF_FLAG_FORCE_VALU);
    // unit-resident kernel: as many cooperating workgroups per unit as it takes to fill the
    // chip, more if one workgroup's share of the codes would not fit its LDS
    const bool stash = !(p->flags & LF_FLAG_ATTENTION_ONLY);
    int S = (cfg->flags & LF_FLAG_FORCE_UNIT) ? 1 : unit_mfma_splits(p->units, p->N);
    while (S < 8 && unit_mfma_lds_bytes(p->N, p->G, stash, S) > kUnitLdsLimit) ++S;
    const bool fits = unit_mfma_lds_bytes(p->N, p->G, stash, S) <= kUnitLdsLimit;
    p->unit_S = S;
    p->use_unit = p->use_mfma && fits && !(cfg->flags & LF_FLAG_FORCE_SPLIT);
    if (p->use_unit && S > p->C) p->C = S; // the partial buffers are shared with the split path
}

static Layout layout_of(const Plan &p)
{
    Layout l;
    l.n_regions = 0;
    const size_t esz = p.dtype == LF_F32 ? 4 : 2;
    size_t off = 0;
    auto take = [&](const char *name, size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        l.region_name[l.n_regions] = name; l.region_off[l.n_regions] = o; l.region_bytes[l.n_regions] = bytes;
        ++l.n_regions;
        return o;
    };
    l.off_pending = take("pending", sizeof(int32_t) * p.units);
    l.off_arrive = take("arrive", sizeof(int32_t) * p.units);
    l.off_hole = take("first_hole", sizeof(int32_t) * p.units);
    l.off_q = take("q_last", esz * (size_t)p.B * p.Hq * p.D);
    l.off_part_m = take("part_m", sizeof(float) * (size_t)p.units * p.C * kMaxGroup);
    l.off_part_l = take("part_l", sizeof(float) * (size_t)p.units * p.C * kMaxGroup);
    l.off_part_o = take("part_o", sizeof(float) * (size_t)p.units * p.C * p.G * p.D);
    l.off_fin_m = take("fin_m", sizeof(float) * (size_t)p.units * p.G);
    l.off_fin_l = take("fin_l", sizeof(float) * (size_t)p.units * p.G);
    // per-slot screening data in device memory: bf16 stash on the split path, 1-byte code
    // dumps when several workgroups share a unit, nothing when one workgroup owns it
    const bool stash = !(p.flags & LF_FLAG_ATTENTION_ONLY) && !(p.use_unit && p.unit_S == 1);
    const size_t per_slot = p.use_unit ? 1 : sizeof(uint16_t);
    l.off_stash_w = take("stash_w", stash ? per_slot * (size_t)p.units * p.ntiles * p.G * kTile : 0);
    l.off_stash_m = take("stash_m", stash ? sizeof(float) * (size_t)p.units * p.ntiles * p.G : 0);
    // per-slot side array: log2 ||v||_1 for the matrix-core kernels, validity under an explicit mask for all
    l.off_lu = take("lu", !(p.flags & LF_FLAG_ATTENTION_ONLY) ? sizeof(float) * (size_t)p.units * p.ntiles * kTile : 0);
    int la = 0, ca = 0;
    if (p.unfused) unfused_geometry(p.units, p.N, &la, &ca);
    l.off_acc = take("acc", p.unfused ? sizeof(float) * (size_t)p.units * p.ntiles * kTile : 0);
    l.off_acc_part_v = take("acc_part_v", sizeof(float) * (size_t)p.units * ca);
    l.off_acc_part_i = take("acc_part_i", sizeof(int32_t) * (size_t)p.units * ca);
    l.total = off;
    return l;
}

} // namespace lf

struct longflow_cache {
    uint32_t magic;
    lf::Plan plan;
    int count;         // valid slots
    bool has_pending;  // a slot for the next token is known on the device
    bool stepped;      // at least one decode step ran (scores are defined)
    std::vector<hipEvent_t> prof_events; // 2 per recorded step while profiling
    int prof_cap = 0, prof_used = 0;
    int groups = 0;    // live groups this cache is a member of
};

static const uint32_t kMagic = 0x4c46434bu;
static const uint32_t kGroupMagic = 0x4c464752u;

struct longflow_group {
    uint32_t magic;
    std::vector<longflow_cache *> members;
    void *table; // device: one kernel-argument entry per member
};

using namespace lf;

static longflow_cache *checked(longflow_cache_t *c)
{
    return (c && c->magic == kMagic) ? c : nullptr;
}

extern "C" {

size_t longflow_workspace_bytes(const lf_config *cfg)
{
    if (validate(cfg) != LF_OK) return 0;
    Plan p;
    fill_plan(cfg, &p);
    return layout_of(p).total;
}

int longflow_workspace_regions(const lf_config *cfg, lf_region *regions, int32_t max_regions, int32_t *n_regions)
{
    if (!n_regions) return fail(LF_ERR_INVALID_ARG, "n_regions is NULL");
    *n_regions = 0;
    const int rc = validate(cfg);
    if (rc != LF_OK) return rc;
    Plan p;
    fill_plan(cfg, &p);
    const Layout l = layout_of(p);
    *n_regions = l.n_regions;
    if (!regions) return LF_OK;
    if (max_regions < l.n_regions) return fail(LF_ERR_INVALID_ARG, "%d regions, room for %d", l.n_regions, max_regions);
    for (int i = 0; i < l.n_regions; ++i) {
        memset(&regions[i], 0, sizeof(regions[i]));
        strncpy(regions[i].name, l.region_name[i], sizeof(regions[i].name) - 1);
        regions[i].offset = l.region_off[i];
        regions[i].bytes = l.region_bytes[i];
    }
    return LF_OK;
}

int longflow_init_cache(longflow_cache_t **out, const lf_config *cfg, void *k_cache, void *v_cache,
                        const void *k_init, const void *v_init, int32_t n_init, void *workspace,
                        size_t workspace_bytes, void *hip_stream)
{
    if (!out) return fail(LF_ERR_INVALID_ARG, "out is NULL");
    *out = nullptr;
    int rc = validate(cfg);
    if (rc != LF_OK) return rc;
    if (!k_cache || !v_cache) return fail(LF_ERR_INVALID_ARG, "k_cache/v_cache is NULL");
    if (n_init < 0 || n_init > cfg->budget)
        return fail(LF_ERR_INVALID_ARG, "n_init %d outside [0, %d]", n_init, cfg->budget);
    if (n_init > 0 && (!k_init || !v_init)) return fail(LF_ERR_INVALID_ARG, "k_init/v_init is NULL");
    if (!workspace) return fail(LF_ERR_INVALID_ARG, "workspace is NULL");
    if (((uintptr_t)workspace & 255u) || ((uintptr_t)k_cache & 15u) || ((uintptr_t)v_cache & 15u))
        return fail(LF_ERR_INVALID_ARG, "workspace must be 256-byte, caches 16-byte aligned");
    Plan p;
    fill_plan(cfg, &p);
    if (p.max_free && !p.use_unit)
        return fail(LF_ERR_UNSUPPORTED, "MAX_FREE: budget %d x group %d does not fit the fused kernel's LDS", p.N, p.G);
    const Layout l = layout_of(p);
    if (workspace_bytes < l.total)
        return fail(LF_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, l.total);
    char *ws = (char *)workspace;
    p.k_cache = k_cache; p.v_cache = v_cache;
    p.pending = (int32_t *)(ws + l.off_pending);
    p.arrive = (int32_t *)(ws + l.off_arrive);
    p.first_hole = (int32_t *)(ws + l.off_hole);
    p.q_last = ws + l.off_q;
    p.part_m = (float *)(ws + l.off_part_m);
    p.part_l = (float *)(ws + l.off_part_l);
    p.part_o = (float *)(ws + l.off_part_o);
    p.fin_m = (float *)(ws + l.off_fin_m);
    p.fin_l = (float *)(ws + l.off_fin_l);
    p.stash_w = (uint16_t *)(ws + l.off_stash_w);
    p.stash_m = (float *)(ws + l.off_stash_m);
    p.lu = (float *)(ws + l.off_lu);
    p.acc = (float *)(ws + l.off_acc);
    p.acc_part_v = (float *)(ws + l.off_acc_part_v);
    p.acc_part_i = (int32_t *)(ws + l.off_acc_part_i);

    hipStream_t s = (hipStream_t)hip_stream;
    {   // set-up for longflow_evict_lowest_static: its device array's address on this GPU is
        // resolved here, so that the call itself (possibly made where nothing may allocate or
        // query the runtime) only looks it up
        hipError_t e = static_score_scratch(nullptr);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "static scratch address: %s", hipGetErrorString(e));
    }
    if (n_init > 0) {
        const size_t esz = p.dtype == LF_F32 ? 4 : 2;
        const size_t row = esz * p.D;
        hipError_t e = hipMemcpy2DAsync(k_cache, row * p.N, k_init, row * n_init, row * n_init, p.units,
                                        hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess)
            e = hipMemcpy2DAsync(v_cache, row * p.N, v_init, row * n_init, row * n_init, p.units,
                                 hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "prefill copy: %s", hipGetErrorString(e));
    }
    if (n_init > 0 && p.use_mfma && !(p.flags & LF_FLAG_ATTENTION_ONLY)) {
        hipError_t e = launch_l1norms(p, n_init, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "value-norm init: %s", hipGetErrorString(e));
    }
    {
        hipError_t e = launch_fill_i32(p.arrive, p.units, 0, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "counter init: %s", hipGetErrorString(e));
    }
    if (p.unfused) { // prefilled rows start with no attention on their books
        hipError_t e = launch_fill_i32((int32_t *)p.acc, p.units * p.ntiles * kTile, 0, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "accumulator init: %s", hipGetErrorString(e));
    }
    const bool filling = n_init < p.N;
    if (filling) {
        hipError_t e = launch_fill_i32(p.pending, p.units, n_init, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "pending init: %s", hipGetErrorString(e));
    }
    longflow_cache *c = new longflow_cache;
    c->magic = kMagic;
    c->plan = p;
    c->count = n_init;
    c->has_pending = filling;
    c->stepped = false;
    *out = c;
    g_err[0] = 0;
    return LF_OK;
}

int longflow_decode_step(longflow_cache_t *cache, const void *q, const void *k_new, const void *v_new,
                         void *out, int32_t *evict_idx, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    const Plan &p = c->plan;
    const bool attention_only = (p.flags & LF_FLAG_ATTENTION_ONLY) && !p.unfused;
    if (!q || !out) return fail(LF_ERR_INVALID_ARG, "q/out is NULL");
    if (!attention_only && (!k_new || !v_new)) return fail(LF_ERR_INVALID_ARG, "k_new/v_new is NULL");
    if (((uintptr_t)q & 15u) || ((uintptr_t)out & 15u))
        return fail(LF_ERR_INVALID_ARG, "q/out must be 16-byte aligned");
    if (p.unfused && (((uintptr_t)k_new & 15u) || ((uintptr_t)v_new & 15u)))
        return fail(LF_ERR_INVALID_ARG, "k_new/v_new must be 16-byte aligned");
    int n;
    if (attention_only) {
        if (c->count < 1) return fail(LF_ERR_STATE, "attention over an empty cache");
        n = c->count;
    } else {
        if (!c->has_pending)
            return fail(LF_ERR_STATE, "cache is full and no slot is pending: call longflow_set_pending");
        n = c->count < p.N ? c->count + 1 : p.N;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    hipEvent_t *ev = nullptr;
    if (c->prof_used < c->prof_cap) ev = &c->prof_events[2 * (size_t)c->prof_used++];
    if (ev) (void)hipEventRecord(ev[0], s);
    hipError_t e;
    if (p.unfused) {
        const StepIo io = {q, k_new, v_new, out, evict_idx};
        e = launch_unfused_step(p, io, n, s);
    } else if (p.use_unit) {
        e = launch_unit_mfma(p, q, k_new, v_new, n, out, evict_idx, s);
    } else {
        const StepIo io = {q, k_new, v_new, out, evict_idx};
        e = p.use_mfma ? launch_split_mfma(p, io, n, s) : p.use_mfma32 ? launch_split_mfma32(p, io, n, s) : launch_split_valu(p, io, n, s);
    }
    if (e != hipSuccess) return fail(LF_ERR_HIP, "decode launch: %s", hipGetErrorString(e));
    if (ev) (void)hipEventRecord(ev[1], s);
    c->count = n;
    c->stepped = true;
    return LF_OK;
}

int longflow_fill_steps(longflow_cache_t *cache, int32_t T, const void *q, const void *k_new, const void *v_new,
                        void *out, int32_t *evict_idx, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    const Plan &p = c->plan;
    if (p.unfused) return fail(LF_ERR_UNSUPPORTED, "the unfused comparison path has no bulk fill");
    if (p.flags & LF_FLAG_ATTENTION_ONLY) return fail(LF_ERR_UNSUPPORTED, "an attention-only cache takes no tokens");
    if (!q || !k_new || !v_new || !out) return fail(LF_ERR_INVALID_ARG, "q/k_new/v_new/out is NULL");
    if (((uintptr_t)q & 15u) || ((uintptr_t)out & 15u) || ((uintptr_t)k_new & 15u) || ((uintptr_t)v_new & 15u))
        return fail(LF_ERR_INVALID_ARG, "q/k_new/v_new/out must be 16-byte aligned");
    if (T < 1) return fail(LF_ERR_INVALID_ARG, "T = %d", T);
    if (!c->has_pending)
        return fail(LF_ERR_STATE, "cache is full and no slot is pending: call longflow_set_pending");
    hipStream_t s = (hipStream_t)hip_stream;
    const size_t esz = p.dtype == LF_F32 ? 4 : 2;
    const size_t q_step = esz * (size_t)p.B * p.Hq * p.D, kv_step = esz * (size_t)p.B * p.Hkv * p.D;
    // The tokens that find a free slot go in bulk where that pays, all but the last of them: that
    // one takes the ordinary step, which also leaves what longflow_scores needs and makes the
    // eviction decision if the cache is now full.  Tokens beyond the free slots are ordinary
    // evicting steps, issued back to back.
    const int room = p.masked ? 0 : p.N - c->count;
    const int Tfill = std::min<int>(T, room);
    int Tb = 0;
    // (the batched kernel keeps a softmax reference: a max-free cache takes its tokens as single steps)
    if (p.use_mfma && !p.max_free && Tfill - 1 >= fill_tokens_per_pass(p.G)) {
        Tb = Tfill - 1;
        // one workgroup per (unit, group of tokens): keep each launch's grid below 2^30 workgroups
        const long long per_launch = std::max(1ll, (1ll << 30) / p.units) * fill_tokens_per_pass(p.G);
        // (a launch failure leaves the cache at the last chunk that went through: count and the
        // pending slot are advanced chunk by chunk)
        const int n0 = c->count;
        for (long long done = 0; done < Tb; done += per_launch) {
            const int Tc = (int)std::min<long long>(per_launch, Tb - done);
            hipError_t e = launch_fill_bulk(p, (const char *)q + done * q_step, (const char *)k_new + done * kv_step,
                                            (const char *)v_new + done * kv_step, (char *)out + done * q_step, n0 + (int)done, Tc, s);
            if (e == hipSuccess) e = launch_fill_i32(p.pending, p.units, n0 + (int)done + Tc, s);
            if (e != hipSuccess) return fail(LF_ERR_HIP, "bulk fill launch: %s", hipGetErrorString(e));
            c->count = n0 + (int)done + Tc;
        }
    }
    for (int t = Tb; t < T; ++t) {
        const int rc = longflow_decode_step(cache, (const char *)q + t * q_step, (const char *)k_new + t * kv_step,
                                            (const char *)v_new + t * kv_step, (char *)out + t * q_step, evict_idx, hip_stream);
        if (rc != LF_OK) return rc;
    }
    return LF_OK;
}

size_t longflow_compress_scratch_bytes(const lf_config *cfg, int32_t T, int32_t W)
{
    if (validate(cfg) != LF_OK) return 0;
    if (T < 1 || T > (1 << 24) || W < 1 || W > T) return 0;
    const int G = cfg->q_heads / cfg->kv_heads;
    if ((long long)W * G > 4096) return 0;
    return compress_layout(cfg->batch * cfg->kv_heads, G, T, W, cfg->budget).total;
}

int longflow_compress_prompt(longflow_cache_t *cache, int32_t T, int32_t W, int32_t keep, int32_t pool,
                             const void *q_window, const void *k_prompt, const void *v_prompt, void *scratch,
                             size_t scratch_bytes, float *pooled, int32_t *kept, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    const Plan &p = c->plan;
    if (p.unfused) return fail(LF_ERR_UNSUPPORTED, "the unfused comparison path has no prompt compression");
    if (p.flags & LF_FLAG_ATTENTION_ONLY) return fail(LF_ERR_UNSUPPORTED, "an attention-only cache takes no tokens");
    if (!p.use_mfma) return fail(LF_ERR_UNSUPPORTED, "prompt compression needs bf16, head_dim 128 and the matrix-core kernels");
    if (c->count != 0 || p.masked || c->stepped)
        return fail(LF_ERR_STATE, "prompt compression starts from an empty cache (this one holds %d rows)", c->count);
    if (c->groups > 0) return fail(LF_ERR_STATE, "cache is a member of a live group");
    if (!q_window || !k_prompt || !v_prompt) return fail(LF_ERR_INVALID_ARG, "q_window/k_prompt/v_prompt is NULL");
    if (((uintptr_t)q_window & 15u) || ((uintptr_t)k_prompt & 15u) || ((uintptr_t)v_prompt & 15u))
        return fail(LF_ERR_INVALID_ARG, "q_window/k_prompt/v_prompt must be 16-byte aligned");
    if (T < 1 || T > (1 << 24)) return fail(LF_ERR_INVALID_ARG, "T = %d outside [1, 2^24]", T);
    if (W < 1 || keep < W || keep > T) return fail(LF_ERR_INVALID_ARG, "need 1 <= W <= keep <= T (W %d, keep %d, T %d)", W, keep, T);
    if (keep > p.N) return fail(LF_ERR_INVALID_ARG, "keep %d exceeds the budget %d", keep, p.N);
    if (pool < 1 || !(pool & 1) || pool > 1023) return fail(LF_ERR_INVALID_ARG, "pool %d is not an odd number in [1, 1023]", pool);
    if ((long long)W * p.G > 4096) return fail(LF_ERR_UNSUPPORTED, "window %d x group %d: more than 4096 query columns", W, p.G);
    if ((long long)p.units * T >= (1ll << 31) / 16) // grids of one 16-lane row per element stay valid launches
        return fail(LF_ERR_UNSUPPORTED, "batch*kv_heads*T >= 2^27");
    const CompressLayout l = compress_layout(p.units, p.G, T, W, p.N);
    if (!scratch || ((uintptr_t)scratch & 255u)) return fail(LF_ERR_INVALID_ARG, "scratch is NULL or not 256-byte aligned");
    if (scratch_bytes < l.total) return fail(LF_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, l.total);
    hipStream_t s = (hipStream_t)hip_stream;
    hipError_t e = launch_compress_prompt(p, T, W, keep, pool, q_window, k_prompt, v_prompt, scratch, s);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "prompt compression launch: %s", hipGetErrorString(e));
    if (pooled && T > W) {
        e = hipMemcpyAsync(pooled, (char *)scratch + l.off_pooled, sizeof(float) * (size_t)p.units * (T - W), hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "pooled votes copy: %s", hipGetErrorString(e));
    }
    if (kept) {
        e = hipMemcpyAsync(kept, (char *)scratch + l.off_kept, sizeof(int32_t) * (size_t)p.units * keep, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "kept rows copy: %s", hipGetErrorString(e));
    }
    c->count = keep;
    c->has_pending = keep < p.N;
    if (c->has_pending) {
        e = launch_fill_i32(p.pending, p.units, keep, s);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "pending init: %s", hipGetErrorString(e));
    }
    return LF_OK;
}

int longflow_scores(longflow_cache_t *cache, float *scores, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (!scores) return fail(LF_ERR_INVALID_ARG, "scores is NULL");
    if (!c->stepped) return fail(LF_ERR_STATE, "no decode step has run yet");
    if (c->plan.unfused) { // the books themselves; slots never filled still hold their initial 0
        hipError_t e = launch_unfused_scores(c->plan, scores, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "accumulator copy: %s", hipGetErrorString(e));
        return LF_OK;
    }
    if (c->plan.flags & LF_FLAG_ATTENTION_ONLY)
        return fail(LF_ERR_STATE, "scores are not defined for an attention-only cache");
    hipError_t e = launch_scores(c->plan, c->count, scores, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "scores launch: %s", hipGetErrorString(e));
    return LF_OK;
}

int longflow_set_pending(longflow_cache_t *cache, const int32_t *slots, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (!slots) return fail(LF_ERR_INVALID_ARG, "slots is NULL");
    if (c->count < c->plan.N)
        return fail(LF_ERR_STATE, "cache is still filling (%d of %d): the next slot is fixed", c->count,
                    c->plan.N);
    hipError_t e = hipMemcpyAsync(c->plan.pending, slots, sizeof(int32_t) * c->plan.units,
                                  hipMemcpyDeviceToDevice, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "set_pending copy: %s", hipGetErrorString(e));
    c->has_pending = true;
    return LF_OK;
}

int longflow_plan_info(const lf_config *cfg, lf_plan_info *info)
{
    if (!info) return fail(LF_ERR_INVALID_ARG, "info is NULL");
    memset(info, 0, sizeof(*info));
    const int rc = validate(cfg);
    if (rc != LF_OK) return rc;
    Plan p;
    fill_plan(cfg, &p);
    if (p.use_unit) {
        const int len = unit_mfma_split_len(p.N, p.unit_S);
        info->path = LF_PATH_UNIT_MFMA;
        info->workgroups_per_unit = (p.N + len - 1) / len;
        info->slots_per_workgroup = len;
        info->launches_per_step = 1;
        info->threads_per_workgroup = 512;
        info->lds_bytes = (uint32_t)unit_mfma_lds_bytes(p.N, p.G, !(p.flags & LF_FLAG_ATTENTION_ONLY), p.unit_S);
    } else {
        info->path = p.use_mfma ? LF_PATH_SPLIT_MFMA : p.use_mfma32 ? LF_PATH_SPLIT_MFMA_F32 : LF_PATH_SPLIT_VALU;
        info->workgroups_per_unit = (p.N + p.L - 1) / p.L;
        info->slots_per_workgroup = p.L;
        info->launches_per_step =
            (info->workgroups_per_unit == 1 || (long long)p.units * info->workgroups_per_unit <= 256) ? 1 : 2;
        info->threads_per_workgroup = 256;
        info->lds_bytes = 0;
    }
    if (p.unfused) info->launches_per_step += 3; // insert, accumulate, decide around the attention kernel
    return LF_OK;
}

size_t longflow_group_workspace_bytes(int32_t n_caches)
{
    if (n_caches < 1) return 0;
    return align_up(std::max(unit_mfma_table_entry_bytes(), split_table_entry_bytes()) * (size_t)n_caches, 256);
}

int longflow_group_create(longflow_group_t **group, longflow_cache_t *const *caches, int32_t n_caches,
                          void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!group) return fail(LF_ERR_INVALID_ARG, "group is NULL");
    *group = nullptr;
    if (!caches || n_caches < 1) return fail(LF_ERR_INVALID_ARG, "no caches given");
    if (!workspace || ((uintptr_t)workspace & 255u))
        return fail(LF_ERR_INVALID_ARG, "workspace is NULL or not 256-byte aligned");
    if (workspace_bytes < longflow_group_workspace_bytes(n_caches))
        return fail(LF_ERR_WORKSPACE, "group workspace has %zu bytes, %zu needed", workspace_bytes,
                    longflow_group_workspace_bytes(n_caches));
    std::vector<longflow_cache *> members;
    for (int i = 0; i < n_caches; ++i) {
        longflow_cache *c = checked(caches[i]);
        if (!c) return fail(LF_ERR_STATE, "member %d: invalid or destroyed cache handle", i);
        if (c->plan.unfused) return fail(LF_ERR_UNSUPPORTED, "member %d: the unfused comparison path has no grouped launch", i);
        if (c->plan.max_free) return fail(LF_ERR_UNSUPPORTED, "member %d: the max-free variant has no grouped launch", i);
        for (longflow_cache *m : members)
            if (m == c) return fail(LF_ERR_INVALID_ARG, "member %d appears twice", i);
        const Plan &a = c->plan, &b = (members.empty() ? c : members[0])->plan;
        if (a.B != b.B || a.Hq != b.Hq || a.Hkv != b.Hkv || a.D != b.D || a.N != b.N || a.dtype != b.dtype ||
            a.flags != b.flags)
            return fail(LF_ERR_INVALID_ARG, "member %d differs from member 0 in its configuration", i);
        if (a.masked != b.masked)
            return fail(LF_ERR_STATE, "member %d differs from member 0 in whether a mask is in force", i);
        members.push_back(c);
    }
    {   // one grid serves all members: it must stay a valid launch
        const Plan &p0 = members[0]->plan;
        const long long per_cache = (long long)p0.units * std::max(p0.C, p0.unit_S);
        if (per_cache * n_caches >= (1ll << 31))
            return fail(LF_ERR_UNSUPPORTED, "%d caches of %d units are more workgroups than one launch takes", n_caches, p0.units);
    }
    // one entry per member, in the layout of the kernel family its plan uses
    const bool unit = members[0]->plan.use_unit;
    const size_t eb = unit ? unit_mfma_table_entry_bytes() : split_table_entry_bytes();
    if (eb > kTableEntryMax) return fail(LF_ERR_UNSUPPORTED, "table entry of %zu bytes", eb);
    for (int i = 0; i < n_caches; ++i) { // each entry travels as a kernel argument: asynchronous, nothing to keep alive
        char entry[kTableEntryMax];
        if (unit) unit_mfma_table_entry(members[i]->plan, entry);
        else      split_table_entry(members[i]->plan, entry);
        hipError_t e = launch_table_entry((char *)workspace + eb * i, entry, eb, (hipStream_t)hip_stream);
        if (e != hipSuccess) return fail(LF_ERR_HIP, "group table write: %s", hipGetErrorString(e));
    }
    longflow_group *g = new longflow_group;
    g->magic = kGroupMagic;
    g->members = members;
    g->table = workspace;
    for (longflow_cache *m : members) ++m->groups;
    *group = g;
    return LF_OK;
}

int longflow_group_decode_step(longflow_group_t *group, const void *q, const void *k_new, const void *v_new,
                               void *out, int32_t *evict_idx, void *hip_stream)
{
    if (!group || group->magic != kGroupMagic) return fail(LF_ERR_STATE, "invalid or destroyed group handle");
    longflow_cache *c0 = group->members[0];
    const Plan &p = c0->plan;
    const bool attention_only = p.flags & LF_FLAG_ATTENTION_ONLY;
    if (!q || !out) return fail(LF_ERR_INVALID_ARG, "q/out is NULL");
    if (!attention_only && (!k_new || !v_new)) return fail(LF_ERR_INVALID_ARG, "k_new/v_new is NULL");
    if (((uintptr_t)q & 15u) || ((uintptr_t)out & 15u))
        return fail(LF_ERR_INVALID_ARG, "q/out must be 16-byte aligned");
    for (size_t i = 0; i < group->members.size(); ++i) {
        const longflow_cache *c = group->members[i];
        if (c->count != c0->count)
            return fail(LF_ERR_STATE, "member %zu holds %d rows, member 0 holds %d", i, c->count, c0->count);
        if (c->plan.masked != c0->plan.masked)
            return fail(LF_ERR_STATE, "member %zu differs from member 0 in whether a mask is in force", i);
        if (!attention_only && !c->has_pending)
            return fail(LF_ERR_STATE, "member %zu is full and no slot is pending: call longflow_set_pending", i);
    }
    int n;
    if (attention_only) {
        if (c0->count < 1) return fail(LF_ERR_STATE, "attention over an empty cache");
        n = c0->count;
    } else {
        n = c0->count < p.N ? c0->count + 1 : p.N;
    }
    hipStream_t s = (hipStream_t)hip_stream;
    const int nc = (int)group->members.size();
    const StepIo io = {q, k_new, v_new, out, evict_idx};
    hipError_t e;
    if (p.use_unit) e = launch_unit_mfma_group(p, io, n, group->table, nc, s);
    else if (p.use_mfma) e = launch_split_mfma(p, io, n, s, group->table, nc);
    else if (p.use_mfma32) e = launch_split_mfma32(p, io, n, s, group->table, nc);
    else e = launch_split_valu(p, io, n, s, group->table, nc);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "group decode launch: %s", hipGetErrorString(e));
    for (longflow_cache *c : group->members) {
        c->count = n;
        c->stepped = true;
    }
    return LF_OK;
}

int longflow_group_destroy(longflow_group_t *group)
{
    if (!group || group->magic != kGroupMagic) return fail(LF_ERR_STATE, "invalid or destroyed group handle");
    for (longflow_cache *m : group->members) --m->groups;
    group->magic = 0;
    delete group;
    return LF_OK;
}

int longflow_set_mask(longflow_cache_t *cache, const uint8_t *mask, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (!mask) return fail(LF_ERR_INVALID_ARG, "mask is NULL");
    if (c->plan.unfused) return fail(LF_ERR_UNSUPPORTED, "the unfused comparison path takes no mask");
    if (c->plan.flags & LF_FLAG_ATTENTION_ONLY)
        return fail(LF_ERR_UNSUPPORTED, "an attention-only cache takes no mask");
    if (c->plan.max_free) return fail(LF_ERR_UNSUPPORTED, "the max-free variant takes no mask");
    hipError_t e = launch_set_mask(c->plan, mask, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "mask launch: %s", hipGetErrorString(e));
    c->plan.masked = true;
    c->count = c->plan.N; // every step now looks at all N slots
    return LF_OK;
}

int longflow_get_mask(longflow_cache_t *cache, uint8_t *mask, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (!mask) return fail(LF_ERR_INVALID_ARG, "mask is NULL");
    hipError_t e = launch_get_mask(c->plan, c->count, mask, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "mask read-back launch: %s", hipGetErrorString(e));
    return LF_OK;
}

size_t longflow_evict_scratch_bytes(const lf_config *cfg)
{
    if (validate(cfg) != LF_OK) return 0;
    return align_up(sizeof(double) * (size_t)cfg->batch * cfg->kv_heads * cfg->budget, 256);
}

int longflow_evict_lowest(longflow_cache_t *cache, int32_t k, void *scratch, size_t scratch_bytes,
                          int32_t *evicted, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    const Plan &p = c->plan;
    if (p.unfused) return fail(LF_ERR_UNSUPPORTED, "the unfused comparison path evicts one slot per step only");
    if (p.flags & LF_FLAG_ATTENTION_ONLY) return fail(LF_ERR_UNSUPPORTED, "an attention-only cache evicts nothing");
    if (p.max_free) return fail(LF_ERR_UNSUPPORTED, "the max-free variant has no batch eviction (it takes no mask)");
    if (!c->stepped) return fail(LF_ERR_STATE, "no decode step has run yet: there are no scores");
    if (k < 1 || k >= p.N) return fail(LF_ERR_INVALID_ARG, "k = %d outside [1, %d)", k, p.N);
    const size_t need = sizeof(double) * (size_t)p.units * p.N;
    if (!scratch || ((uintptr_t)scratch & 7u)) return fail(LF_ERR_INVALID_ARG, "scratch is NULL or misaligned");
    if (scratch_bytes < need) return fail(LF_ERR_WORKSPACE, "scratch has %zu bytes, %zu needed", scratch_bytes, need);
    hipError_t e = launch_evict_lowest(p, c->count, k, (double *)scratch, evicted, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "batch eviction launch: %s", hipGetErrorString(e));
    c->plan.masked = true;
    c->count = p.N;
    c->has_pending = true; // every unit now has a hole, and its lowest one is pending
    return LF_OK;
}

int longflow_evict_lowest_static(longflow_cache_t *cache, int32_t k, int32_t *evicted, void *hip_stream)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    const Plan &p = c->plan;
    if (p.unfused) return fail(LF_ERR_UNSUPPORTED, "the unfused comparison path evicts one slot per step only");
    if (p.flags & LF_FLAG_ATTENTION_ONLY) return fail(LF_ERR_UNSUPPORTED, "an attention-only cache evicts nothing");
    if (p.max_free) return fail(LF_ERR_UNSUPPORTED, "the max-free variant has no batch eviction (it takes no mask)");
    if ((size_t)p.units * p.N > kStaticScoreSlots)
        return fail(LF_ERR_WORKSPACE, "batch*kv_heads*budget = %zu exceeds the %zu slots of the built-in scratch: "
                    "use longflow_evict_lowest with a scratch buffer of your own", (size_t)p.units * p.N, kStaticScoreSlots);
    if (!c->stepped) return fail(LF_ERR_STATE, "no decode step has run yet: there are no scores");
    if (k < 1 || k >= p.N) return fail(LF_ERR_INVALID_ARG, "k = %d outside [1, %d)", k, p.N);
    double *scores = nullptr;
    hipError_t e = static_score_scratch(&scores);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "static scratch address: %s", hipGetErrorString(e));
    e = launch_evict_lowest(p, c->count, k, scores, evicted, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(LF_ERR_HIP, "batch eviction launch: %s", hipGetErrorString(e));
    c->plan.masked = true;
    c->count = p.N;
    c->has_pending = true;
    return LF_OK;
}

static void drop_events(longflow_cache *c)
{
    for (hipEvent_t e : c->prof_events) (void)hipEventDestroy(e);
    c->prof_events.clear();
    c->prof_cap = c->prof_used = 0;
}

int longflow_profile_begin(longflow_cache_t *cache, int32_t max_steps)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (max_steps < 1 || max_steps > (1 << 20)) return fail(LF_ERR_INVALID_ARG, "max_steps out of range");
    drop_events(c);
    c->prof_events.resize(2 * (size_t)max_steps);
    for (size_t i = 0; i < c->prof_events.size(); ++i) {
        hipError_t e = hipEventCreateWithFlags(&c->prof_events[i], hipEventDisableSystemFence);
        if (e != hipSuccess) {
            c->prof_events.resize(i);
            drop_events(c);
            return fail(LF_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e));
        }
    }
    c->prof_cap = max_steps;
    c->prof_used = 0;
    return LF_OK;
}

int longflow_profile_end(longflow_cache_t *cache, float *kernel_ms, int32_t *steps)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (!kernel_ms || !steps) return fail(LF_ERR_INVALID_ARG, "kernel_ms/steps is NULL");
    *kernel_ms = 0.f;
    *steps = c->prof_used;
    int rc = LF_OK;
    for (int i = 0; i < c->prof_used && rc == LF_OK; ++i) {
        hipEvent_t *ev = &c->prof_events[2 * (size_t)i];
        hipError_t e = hipEventSynchronize(ev[1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
        *kernel_ms += ms;
        if (e != hipSuccess) rc = fail(LF_ERR_HIP, "event timing: %s", hipGetErrorString(e));
    }
    drop_events(c);
    return rc;
}

int longflow_valid_count(const longflow_cache_t *cache)
{
    return (cache && cache->magic == kMagic) ? cache->count : -1;
}

int longflow_destroy_cache(longflow_cache_t *cache)
{
    longflow_cache *c = checked(cache);
    if (!c) return fail(LF_ERR_STATE, "invalid or destroyed cache handle");
    if (c->groups > 0) return fail(LF_ERR_STATE, "cache is a member of %d live group(s): destroy them first", c->groups);
    drop_events(c);
    c->magic = 0;
    delete c;
    return LF_OK;
}

const char *longflow_last_error(void) { return g_err; }

} // extern "C"
