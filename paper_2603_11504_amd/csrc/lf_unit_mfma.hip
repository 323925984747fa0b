// Unit-resident fused decode step on the matrix cores (bf16, head_dim 128).
//
// A (batch, KV head) unit is owned for the whole call by S workgroups of 8 waves
// (S = 1 when there are enough units to fill the chip, else up to 8), and every step of
// the path happens in ONE launch with no per-slot intermediate in device memory:
//
//   insert   the wave that will stream the pending slot's tile writes k_new / v_new into it
//   stream   this workgroup's share of the valid slots, once: logits, online softmax,
//            P V (eq. 1), leaving an 8-bit log2 code of ||v_i||_1 * p_h,i per (head, slot)
//            in LDS (eq. 6)
//   merge    the 8 waves' softmax states; with S > 1 the workgroup publishes its partial
//            (m, l, O) and the LAST workgroup of the unit to arrive merges the S partials
//   evict    screen every slot with the codes (bounds within a factor 2^(1/8)), re-score the
//            few that can still be the minimum exactly in double precision, argmin
//   output   normalise, round to bf16
//
// Keeping the per-slot by-products in LDS matters on this chip: even a few percent of HBM
// writes interleaved with the K/V read stream cost a quarter of the read bandwidth.
//
// Cooperation protocol for S > 1 (no workgroup ever waits for one that is not already
// running): each workgroup writes its partial through to the device-wide coherence point,
// waits for its own stores, and bumps arrive[u].  All but the last then write their codes
// to a dump area the same way and bump dumped[u].  The last one merges the partials (the
// partial outputs come in the same batch of loads, the output is stored at once), waits
// (bounded) until S-1 dumps are in -- their authors passed arrive[u] before it did, so they
// are running or done -- and decides the eviction from its own LDS codes plus the dumps,
// which it reads in place (S = 2) or copies into LDS chunk by chunk (S >= 3).  If the
// bounded wait ever expired it would re-score every slot exactly instead of trusting
// incomplete dumps.
#include <algorithm>
#include <cstring>

#include "lf_mfma_stream.h"

namespace lf {

constexpr int kMaxCand = 256; // candidates listed in LDS; more than this falls back to a slow scan

struct UnitArgs {
    uint16_t *Kc, *Vc;                 // caches [units][N][128]
    const uint16_t *q, *k_new, *v_new;
    uint16_t *out, *q_last;
    int32_t *pending, *evict_idx;
    float *fin_m, *fin_l;              // [units][G] reference / denominator of the step
    float *lu;                         // [units][ntiles*16] log2 ||v||_1, position order
    // cooperation of S workgroups per unit (untouched when s_active == 1)
    float *part_m, *part_l, *part_o;   // [units][S][16], [units][S][16], [units][S][G][128]
    int32_t *arrive, *dumped;          // [units], zero between steps
    uint8_t *gcode;                    // [units][G][gstride] dumped codes, absolute positions
    float *gref;                       // [units][ntiles][G] dumped references
    int n, N, G, ntiles;
    int S, s_active, split_len;        // split_len: slots per workgroup, a multiple of 128
    int code_stride, gstride;          // LDS / dump row strides in bytes
    int merge_off;                     // byte offset of the O-merge area in dynamic LDS
    int chunk_len;                     // positions of the other workgroups' dumps the deciding one copies into
                                       // LDS at a time (multiple of 2048; 0: it reads them in place)
    float scale_log2;
};

// One launch over several caches of identical geometry and fill level: the per-cache
// pointers come from a device-resident table of UnitArgs, the step's tensors from base
// pointers with a per-cache stride (in elements).
struct GroupArgs {
    const UnitArgs *table;
    int wgs_per_cache;
    long long q_stride, kv_stride, ev_stride;
};

// Device-scope coherent accesses for the little data that cooperating workgroups exchange.
// Stores write through to the coherence point and loads bypass stale cached copies, so
// publishing needs only "wait for my stores, then bump the counter": no L2 write-back
// (buffer_wbl2) and no invalidate, which on this 8-XCD part cost far more than the
// exchange itself (measured on 128 units x 4096 slots: 160 us with per-thread fences, 70 us
// with one fence pair per workgroup, 58 us with this scheme).
template <typename T> __device__ __forceinline__ void st_agent(T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ T ld_agent(const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// all of this thread's device-scope stores have reached the coherence point
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

__device__ __forceinline__ double wave_sum_f64(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// 2^x for |x| <= 0.5 in double precision: Taylor series of exp(x ln 2), error < 1e-14
__device__ __forceinline__ double exp2_frac_f64(double x)
{
    const double y = x * 0.69314718055994530942;
    double p = 1.0 / 39916800.0;
    p = fma(p, y, 1.0 / 3628800.0);
    p = fma(p, y, 1.0 / 362880.0);
    p = fma(p, y, 1.0 / 40320.0);
    p = fma(p, y, 1.0 / 5040.0);
    p = fma(p, y, 1.0 / 720.0);
    p = fma(p, y, 1.0 / 120.0);
    p = fma(p, y, 1.0 / 24.0);
    p = fma(p, y, 1.0 / 6.0);
    p = fma(p, y, 0.5);
    p = fma(p, y, 1.0);
    p = fma(p, y, 1.0);
    return p;
}

// Exact LongFlowScore of one slot in double precision (eq. 6 with the group's heads
// summed), computed by one wave: 4 lanes per head, 32 channels per lane.
//   qs: the step's query as floats in LDS [16][128]; sM: softmax reference per head
//   (log2 domain); sL: denominator per head.
//   coherent: read the row with device-scope loads (it was written during this launch by
//   another workgroup)
__device__ double exact_score_bf16(const uint16_t *krow, const uint16_t *vrow, const uint16_t (*qs)[128], int G,
                                   const float *sM, const float *sL, int lane, bool coherent)
{
    const int h = lane >> 2, part = lane & 3;
    // ||v||_1: two channels per lane, summed over the wave
    const uint32_t vv = coherent ? ld_agent((const uint32_t *)vrow + lane) : *(const uint32_t *)(vrow + 2 * lane);
    double l1 = fabs((double)bf16_lo(vv)) + fabs((double)bf16_hi(vv));
    l1 = wave_sum_f64(l1);
    // q_h . k over this lane's 32 channels
    double dot = 0.0;
    if (h < G) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            u32x4 kk;
            if (coherent) {
                const uint32_t *kp = (const uint32_t *)(krow + 32 * part + 8 * c);
                kk = u32x4{ld_agent(kp), ld_agent(kp + 1), ld_agent(kp + 2), ld_agent(kp + 3)};
            } else {
                kk = *(const u32x4 *)(krow + 32 * part + 8 * c);
            }
            const u32x4 qq = *(const u32x4 *)(&qs[h][32 * part + 8 * c]);
            dot = fma((double)bf16_lo(qq.x), (double)bf16_lo(kk.x), dot);
            dot = fma((double)bf16_hi(qq.x), (double)bf16_hi(kk.x), dot);
            dot = fma((double)bf16_lo(qq.y), (double)bf16_lo(kk.y), dot);
            dot = fma((double)bf16_hi(qq.y), (double)bf16_hi(kk.y), dot);
            dot = fma((double)bf16_lo(qq.z), (double)bf16_lo(kk.z), dot);
            dot = fma((double)bf16_hi(qq.z), (double)bf16_hi(kk.z), dot);
            dot = fma((double)bf16_lo(qq.w), (double)bf16_lo(kk.w), dot);
            dot = fma((double)bf16_hi(qq.w), (double)bf16_hi(kk.w), dot);
        }
    }
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    double term = 0.0;
    if (h < G && part == 0) {
        const double scale_log2 = 1.4426950408889634074 / 11.313708498984760390; // log2(e) / sqrt(128)
        const double d = dot * scale_log2 - (double)sM[h];
        const double nint = rint(d);
        term = ldexp(exp2_frac_f64(d - nint), (int)nint) / (double)sL[h];
    }
#pragma unroll
    for (int off = 4; off < 64; off <<= 1) term += __shfl_xor(term, off);
    return term * l1;
}

// Explicit-mask mode: the lowest invalid slot of the unit (NaN in the side array), not
// counting the slot this step has just filled (its entry may still read stale here).
// All 512 threads call; true if there is one, then it is in red[0].
__device__ bool fill_lowest_hole(const float *lu_u, int npos, int N, int ins_slot, int *red, int tid, int lane,
                                 int wave)
{
    int best = 0x7fffffff;
    for (int p = tid; p < npos; p += 512) {
        const float x = lu_u[p];
        const int slot = (p & ~15) + slot_of_pos(p & 15);
        if (x != x && slot < N && slot != ins_slot) best = min(best, slot);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) best = min(best, __shfl_xor(best, off));
    if (lane == 0) red[1 + wave] = best;
    __syncthreads();
    if (tid == 0) {
        int b = red[1];
        for (int w = 1; w < 8; ++w) b = min(b, red[1 + w]);
        red[0] = b;
    }
    __syncthreads();
    return red[0] != 0x7fffffff;
}

// value of a unit's dump counter once its codes are no longer trusted (stays negative
// whatever late dumps add to it)
constexpr int kDumpsDistrusted = -(1 << 30);

// COOP: several workgroups may share a unit (s_active can exceed 1)
// GATHER (with COOP): the deciding workgroup copies the others' code dumps into LDS chunk by
// chunk before screening them; without it, it reads them in place, item by item
// MAXFREE (attention only): softmax without a running reference, for A/B measurement
template <bool HILO, int STASH, bool COOP, bool GROUPED, bool MASKED, bool GATHER, bool MAXFREE = false>
__global__ __launch_bounds__(512, 1) void unit_mfma_kernel(const UnitArgs a_in, const GroupArgs ga)
{
    UnitArgs a = a_in;
    int blk = blockIdx.x;
    if (GROUPED) {
        // which cache this workgroup serves; the geometry and the step's scalars are common
        const int ci = blk / ga.wgs_per_cache;
        blk -= ci * ga.wgs_per_cache;
        const UnitArgs *t = ga.table + ci;
        a.Kc = t->Kc; a.Vc = t->Vc; a.q_last = t->q_last; a.pending = t->pending;
        a.fin_m = t->fin_m; a.fin_l = t->fin_l; a.lu = t->lu;
        a.part_m = t->part_m; a.part_l = t->part_l; a.part_o = t->part_o;
        a.arrive = t->arrive; a.dumped = t->dumped; a.gcode = t->gcode; a.gref = t->gref;
        a.q += ci * ga.q_stride;
        a.out += ci * ga.q_stride;
        if (a.k_new) a.k_new += ci * ga.kv_stride;
        if (a.v_new) a.v_new += ci * ga.kv_stride;
        if (a.evict_idx) a.evict_idx += ci * ga.ev_stride;
    }
    constexpr int D = 128, NW = 8, OPAD = D + 4;
    extern __shared__ __align__(16) unsigned char smem[];
    // dynamic LDS: [codes G*code_stride][refs (split_len/16)*G floats]; the O-merge area
    // [NW][G][OPAD] floats starts at merge_off (0 = aliases the codes, used after them)
    uint8_t *ls_code = smem;
    float *ls_ref = (float *)(smem + (size_t)a.G * a.code_stride);
    float *sm_o = (float *)(smem + a.merge_off);
    __shared__ float sm_m[NW][16], sm_l[NW][16], sM[16], sL[16];
    __shared__ float sW[8][16]; // weights of the S partials under the unit-wide reference
    __shared__ float red_f[NW];
    __shared__ double best_v[NW];
    __shared__ int best_i[NW];
    __shared__ __align__(16) uint16_t qs[16][D]; // the query, for the exact re-scoring
    __shared__ int cand_list[kMaxCand];
    __shared__ int cand_count, s_flag;
    __shared__ int red_i[NW + 1];
    __shared__ float exp_tab[256]; // 2^(-c/4) of every code value (screening pass)

    const int n = a.n, N = a.N, G = a.G, s_active = COOP ? a.s_active : 1;
    const int u = blk / s_active, sp = blk % s_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    const int start = sp * a.split_len;
    const int end = min(start + a.split_len, n);
    uint16_t *Ku = a.Kc + (size_t)u * N * D;
    uint16_t *Vu = a.Vc + (size_t)u * N * D;
    const uint16_t *qu = a.q + (size_t)u * G * D;
    float *lu_u = a.lu + (size_t)u * a.ntiles * kTile;
    const bool evicting = (STASH == kStashLds) && n == N;

    // ---- insert (Fig. 2 left): done by the wave that will stream that tile, so that its own
    // later loads of the row are ordered behind the stores.  The row is written through to
    // the device-wide coherence point: with several workgroups per unit, the one that ends
    // up re-scoring candidates may sit on another XCD and must not see the old row.
    const int ins_slot = (STASH != kStashNone) ? a.pending[u] : -1;
    if (STASH != kStashNone) {
        const int slot = ins_slot;
        if (slot >= start && slot < start + a.split_len && slot < N && (((slot - start) / kTile) % NW) == wave) {
            st_agent((uint32_t *)(Ku + (size_t)slot * D) + lane, *((const uint32_t *)(a.k_new + (size_t)u * D) + lane));
            st_agent((uint32_t *)(Vu + (size_t)slot * D) + lane, *((const uint32_t *)(a.v_new + (size_t)u * D) + lane));
            // every 16-lane row sums |v_new| redundantly; lane 0 stores the log2 norm
            const u32x4 vv = *(const u32x4 *)(a.v_new + (size_t)u * D + 8 * r);
            float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                       fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
            a1 = row16_sum(a1);
            if (lane == 0) lu_u[(slot & ~15) + pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }

    // Copies of the query -- LDS for the exact re-scoring, device memory for a later
    // longflow_scores() -- are made now: their load latency hides behind the streaming
    // instead of standing in the serial tail of the kernel.
    if (STASH == kStashLds) {
        for (int i = tid; i < G * D; i += 512) qs[i / D][i % D] = qu[i];
        if (tid < 256) exp_tab[tid] = fast_exp2(-0.25f * (float)tid);
    }
    if (sp == 0)
        for (int i = tid; i < G * D; i += 512) a.q_last[(size_t)u * G * D + i] = qu[i];

    MfmaStreamer<NW, HILO, STASH, MASKED, false, MAXFREE> st;
    st.init(qu, G, lane, a.scale_log2);
    st.Ku = Ku;
    st.Vu = Vu;
    st.start = start;
    st.end = end;
    st.lu_unit = lu_u;
    st.ls_code = ls_code;
    st.ls_ref = ls_ref;
    st.code_stride = a.code_stride;
    st.run(wave);

    // ---- merge the softmax states of the 8 waves
    {
        float l = st.l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) { sm_m[wave][r] = st.m; sm_l[wave][r] = l; }
    }
    if (STASH == kStashLds && tid == 0) cand_count = 0;
    __syncthreads();
    if (tid < 16) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_m[w][tid]);
        float Ls = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) Ls += merge_weight(sm_m[w][tid], M) * sm_l[w][tid];
        sM[tid] = M; // this workgroup's reference and denominator
        sL[tid] = Ls;
    }
    __syncthreads();

    // O of the 8 waves -> LDS, each under this workgroup's reference
    auto stage_o = [&]() {
        float a4[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) a4[v] = merge_weight(sm_m[wave][4 * g + v], sM[4 * g + v]);
        // a lane holds channels 8r .. 8r+7 of heads 4g .. 4g+3: two 16-byte stores per head
        // (single floats at this stride would pile 64 lanes onto a handful of LDS banks)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (4 * g + v < G) { // rows of the G real heads only: the area is sized for them
                float *row = sm_o + ((size_t)wave * G + 4 * g + v) * OPAD + 8 * r;
                *(f32x4 *)row = f32x4{st.oacc[0][v] * a4[v], st.oacc[1][v] * a4[v], st.oacc[2][v] * a4[v], st.oacc[3][v] * a4[v]};
                *(f32x4 *)(row + 4) = f32x4{st.oacc[4][v] * a4[v], st.oacc[5][v] * a4[v], st.oacc[6][v] * a4[v], st.oacc[7][v] * a4[v]};
            }
        }
    };

    bool dumps_ok = true;
    if (COOP && s_active > 1) {
        // ---- publish this workgroup's partial (m, l, O) and count the arrival
        stage_o();
        __syncthreads();
        const size_t pb = (size_t)u * a.S + sp;
        for (int idx = tid; idx < G * D; idx += 512) {
            const int h = idx / D, d = idx % D;
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += sm_o[((size_t)w * G + h) * OPAD + d];
            st_agent(&a.part_o[(pb * G + h) * D + d], acc);
        }
        if (tid < 16) { st_agent(&a.part_m[pb * 16 + tid], sM[tid]); st_agent(&a.part_l[pb * 16 + tid], sL[tid]); }
        wait_stores();
        __syncthreads(); // every thread's partials are visible device-wide before the arrival counts
        if (tid == 0)
            s_flag = (__hip_atomic_fetch_add(&a.arrive[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == s_active - 1);
        __syncthreads();
        if (!s_flag) {
            if (evicting) { // leave the codes where the last workgroup will find them
                const int len = (end - start + kTile - 1) / kTile * kTile; // whole tiles
                for (int i = tid; i < G * (len / 4); i += 512) {
                    const int h = i / (len / 4), j = i % (len / 4);
                    st_agent((uint32_t *)(a.gcode + ((size_t)u * G + h) * a.gstride + start + 4 * j),
                             *(const uint32_t *)(ls_code + (size_t)h * a.code_stride + 4 * j));
                }
                for (int i = tid; i < (len / kTile) * G; i += 512)
                    st_agent(&a.gref[((size_t)u * a.ntiles + start / kTile) * G + i], ls_ref[i]);
                wait_stores();
                __syncthreads();
                if (tid == 0) __hip_atomic_fetch_add(&a.dumped[u], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            return;
        }
        // ---- last arriver: merge the S partials into the unit-wide softmax state and the
        // output.  Device-scope loads are issued in batches (all first, then used): each one
        // is a round trip to the coherence point, and an acquire fence instead (an L2
        // invalidate for the whole XCD) measured slower still.  The partial outputs are
        // fetched in the same batch as the softmax states, so the output costs no trip of
        // its own; it is stored right away (it does not depend on the eviction).
        constexpr int kOutPer = (kMaxGroup * D + 511) / 512;
        float po[kOutPer][8];
#pragma unroll
        for (int k = 0; k < kOutPer; ++k) {
            const int idx = tid + 512 * k;
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2)
                po[k][s2] = (idx < G * D && s2 < s_active)
                                ? ld_agent(&a.part_o[((size_t)u * a.S + s2) * G * D + idx]) : 0.f;
        }
        if (tid < 16) {
            float pm[8], pl[8];
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) {
                pm[s2] = -INFINITY;
                pl[s2] = 0.f;
                if (s2 < s_active) {
                    pm[s2] = ld_agent(&a.part_m[((size_t)u * a.S + s2) * 16 + tid]);
                    pl[s2] = ld_agent(&a.part_l[((size_t)u * a.S + s2) * 16 + tid]);
                }
            }
            float M = -INFINITY;
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) M = fmaxf(M, pm[s2]);
            float Ls = 0.f;
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) {
                const float w = merge_weight(pm[s2], M);
                sW[s2][tid] = w;
                Ls += w * pl[s2];
            }
            sM[tid] = M;
            sL[tid] = Ls;
        }
        if (evicting && tid == 0) { // bounded wait for the S-1 dumps (their authors are running or done)
            // A negative count marks a unit whose wait once ran out: a dump may then have been
            // counted after the counter was cleared, so the counter is never trusted again and
            // every later step re-scores all slots (exact, slower) instead of reading dumps.
            int seen = 0;
            for (int it = 0; it < (1 << 22); ++it) {
                seen = __hip_atomic_load(&a.dumped[u], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (seen >= s_active - 1 || seen < 0) break;
                __builtin_amdgcn_s_sleep(8);
            }
            s_flag = (seen >= s_active - 1);
        }
        __syncthreads();
        if (evicting) dumps_ok = s_flag != 0;
#pragma unroll
        for (int k = 0; k < kOutPer; ++k) {
            const int idx = tid + 512 * k;
            if (idx < G * D) {
                const int h = idx / D;
                float acc = 0.f;
#pragma unroll
                for (int s2 = 0; s2 < 8; ++s2) acc += sW[s2][h] * po[k][s2];
                a.out[(size_t)u * G * D + idx] = (uint16_t)f32_to_bf16_bits(acc / sL[h]);
            }
        }
    }
    if (tid < G) {
        a.fin_m[(size_t)u * G + tid] = sM[tid];
        a.fin_l[(size_t)u * G + tid] = sL[tid];
    }

    // ---- eviction decision (Sec. 3.2 last paragraph; Alg. 1 post-processing)
    if (STASH == kStashLds) {
        if (n < N) {
            if (tid == 0) {
                a.pending[u] = n;
                if (a.evict_idx) a.evict_idx[u] = n;
            }
        } else if (MASKED && fill_lowest_hole(lu_u, a.gstride, N, ins_slot, red_i, tid, lane, wave)) {
            // an invalid slot exists: it takes the next token, nothing is evicted
            if (tid == 0) {
                a.pending[u] = red_i[0];
                if (a.evict_idx) a.evict_idx[u] = red_i[0];
            }
        } else {
            // own codes: per (tile, head) factor that turns a decoded code into a score term
            const int my_tiles = (end - start + kTile - 1) / kTile;
            for (int i = tid; i < my_tiles * G; i += 512) {
                const int h = i % G;
                ls_ref[i] = fast_exp2(kCodeBias + ls_ref[i] - sM[h]) / sL[h];
            }
            // The other workgroups' dumps are screened from LDS too: the deciding workgroup
            // copies them, a chunk of positions at a time, into the LDS that held the O-merge
            // area (dead since the partials were published), every load of a chunk in flight
            // together -- about one trip to the coherence point per chunk, where decoding
            // straight from the dumps pays one per 512 items (measured with 8 workgroups per
            // unit of 16384 slots: screening 67 -> 39 kcycles).  A chunk is a multiple of 2048
            // positions, so that a thread's items (512 apart) fall into chunks as wholes.
            const int own_hi = min(start + a.split_len, a.gstride);
            const int chunk_len = (COOP && GATHER && s_active > 1) ? a.chunk_len : 0;
            uint8_t *rem_code = smem + a.merge_off;
            float *rem_ref = (float *)(rem_code + (size_t)G * chunk_len);
            int chunk_base = 0;
            auto gather_chunk = [&](int cb) {
                constexpr int kBatch = 16;
                // the own range inside the chunk, [lo, hi) relative to cb, is skipped: its codes
                // are in LDS already and its dump is stale
                const int lo = min(max(start - cb, 0), chunk_len), hi = min(max(own_hi - cb, 0), chunk_len);
                const int skip = hi - lo;
                const int top = a.gstride - 8; // last 8-byte word of a dump row
                const int per_h = (chunk_len - skip) / 8;
                const int nw = G * per_h;                             // 8-byte words of codes
                const int tl = lo / kTile, tskip = skip / kTile;
                const int nr = (chunk_len / kTile - tskip) * G;       // references, half as many
                for (int i0 = 0; i0 < nw; i0 += 512 * kBatch) {
                    unsigned long long v[kBatch];
                    float rv[kBatch];
                    int off[kBatch], roff[kBatch];
                    // codes and references of one round are all requested before any is used;
                    // nothing is loaded past the end: device-scope loads are too dear to repeat
#pragma unroll
                    for (int k = 0; k < kBatch; ++k) {
                        const int i = i0 + k * 512 + tid;
                        v[k] = 0;
                        off[k] = 0;
                        if (i < nw) {
                            const int h = i / per_h;
                            int o = 8 * (i % per_h);
                            if (o >= lo) o += skip;
                            off[k] = h * chunk_len + o;
                            v[k] = ld_agent((const unsigned long long *)(a.gcode + ((size_t)u * G + h) * a.gstride + min(cb + o, top)));
                        }
                    }
#pragma unroll
                    for (int k = 0; k < kBatch / 2; ++k) {
                        const int i = i0 / 2 + k * 512 + tid;
                        rv[k] = 0.f;
                        roff[k] = 0;
                        if (i < nr) {
                            int t = i / G;
                            if (t >= tl) t += tskip;
                            roff[k] = t * G + i % G;
                            rv[k] = ld_agent(&a.gref[((size_t)u * a.ntiles + min(cb / kTile + t, a.ntiles - 1)) * G + i % G]);
                        }
                    }
#pragma unroll
                    for (int k = 0; k < kBatch; ++k)
                        if (i0 + k * 512 + tid < nw) *(unsigned long long *)(rem_code + off[k]) = v[k];
#pragma unroll
                    for (int k = 0; k < kBatch / 2; ++k)
                        if (i0 / 2 + k * 512 + tid < nr)
                            rem_ref[roff[k]] = fast_exp2(kCodeBias + rv[k] - sM[roff[k] % G]) / sL[roff[k] % G];
                }
            };
            __syncthreads();
            // Decode every (head, slot) code once.  A decoded term is within 2^(+-1/8) of the
            // true one; code 0 has no upper bound, code 255 no lower bound.  Each thread keeps
            // the lower-bound sums of its slots in registers, the block finds the smallest
            // upper bound, and a slot can be the true minimum only if
            //   2^(-1/8) * lb_sum <= 2^(1/8) * min ub_sum.
            const int items = 4 * ((n + kTile - 1) / kTile); // 4 positions each, whole tiles
            constexpr int kRegIters = 8; // 512 threads x 4 positions x 8 = 16384 slots held in registers
            const int iters = (items + 511) / 512;
            auto decode_item = [&](int item, float *ub4, float *lb4) {
                const int tile = item >> 2;
#pragma unroll
                for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = 0.f;
                // where the item's codes and factors live in LDS, if they do
                const uint8_t *cp = ls_code + 4 * item;
                const float *fp = ls_ref + tile * G;
                int cstride = a.code_stride;
                bool local = true;
                if (COOP) {
                    if (4 * item >= start && 4 * item < own_hi) {
                        cp = ls_code + (4 * item - start);
                        fp = ls_ref + (tile - start / kTile) * G;
                    } else if (GATHER) { // another workgroup's: in the chunk that is in LDS right now
                        const int rp = 4 * item - chunk_base;
                        cp = rem_code + rp;
                        fp = rem_ref + (rp / kTile) * G;
                        cstride = chunk_len;
                    } else {
                        local = false;
                    }
                }
                if (local) {
                    // Common case first: no code of the item sits at a clamp (0x00 or 0xff),
                    // so upper and lower bound share one sum.  The byte tests are the usual
                    // word-at-a-time ones; a hit anywhere sends the item through the exact
                    // two-sided sums below.
                    uint32_t clamped = 0u;
                    for (int h = 0; h < G; ++h) {
                        const uint32_t c4 = *(const uint32_t *)(cp + (size_t)h * cstride);
                        const float f = fp[h];
                        clamped |= ((c4 - 0x01010101u) & ~c4) | ((~c4 - 0x01010101u) & c4);
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            ub4[e] = fmaf(exp_tab[(c4 >> (8 * e)) & 255u], f, ub4[e]);
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) lb4[e] = ub4[e];
                    if (clamped & 0x80808080u) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = 0.f;
                        for (int h = 0; h < G; ++h) {
                            const uint32_t c4 = *(const uint32_t *)(cp + (size_t)h * cstride);
                            const float f = fp[h];
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const uint32_t c = (c4 >> (8 * e)) & 255u;
                                const float d = fast_exp2(-0.25f * (float)c) * f;
                                ub4[e] += (c == 0u) ? INFINITY : d;
                                lb4[e] += (c == 255u) ? 0.f : d;
                            }
                        }
                    }
                } else if (COOP && !GATHER) {
                    // another workgroup's dump, read in place: batch the device-scope loads of
                    // this item, then use them
                    uint32_t c4s[kMaxGroup];
                    float refs[kMaxGroup];
#pragma unroll
                    for (int h = 0; h < kMaxGroup; ++h)
                        if (h < G) {
                            c4s[h] = ld_agent((const uint32_t *)(a.gcode + ((size_t)u * G + h) * a.gstride + 4 * item));
                            refs[h] = ld_agent(&a.gref[((size_t)u * a.ntiles + tile) * G + h]);
                        }
                    // same two forms as above: one sum where no code is clamped, else both
                    uint32_t clamped = 0u;
#pragma unroll
                    for (int h = 0; h < kMaxGroup; ++h) {
                        if (h < G) {
                            refs[h] = fast_exp2(kCodeBias + refs[h] - sM[h]) / sL[h];
                            const uint32_t c4 = c4s[h];
                            clamped |= ((c4 - 0x01010101u) & ~c4) | ((~c4 - 0x01010101u) & c4);
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                ub4[e] = fmaf(exp_tab[(c4 >> (8 * e)) & 255u], refs[h], ub4[e]);
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e) lb4[e] = ub4[e];
                    if (clamped & 0x80808080u) {
#pragma unroll
                        for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = 0.f;
#pragma unroll
                        for (int h = 0; h < kMaxGroup; ++h) {
                            if (h < G) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) {
                                    const uint32_t c = (c4s[h] >> (8 * e)) & 255u;
                                    const float d = fast_exp2(-0.25f * (float)c) * refs[h];
                                    ub4[e] += (c == 0u) ? INFINITY : d;
                                    lb4[e] += (c == 255u) ? 0.f : d;
                                }
                            }
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int slot = ((4 * item) & ~15) + slot_of_pos((4 * item + e) & 15);
                    if (slot >= n) { ub4[e] = INFINITY; lb4[e] = INFINITY; }
                }
            };
            auto list_candidates = [&](int item, const float *lb4, float thr) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (lb4[e] <= thr) {
                        const int k = atomicAdd(&cand_count, 1);
                        if (k < kMaxCand) cand_list[k] = ((4 * item) & ~15) + slot_of_pos((4 * item + e) & 15);
                    }
                }
            };
            auto block_min = [&](float x) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) x = fminf(x, __shfl_xor(x, off));
                if (lane == 0) red_f[wave] = x;
                __syncthreads();
                x = red_f[0];
#pragma unroll
                for (int w = 1; w < NW; ++w) x = fminf(x, red_f[w]);
                return x;
            };
            float ub_min = INFINITY;
            if (!dumps_ok) {
                if (tid == 0) cand_count = kMaxCand + 1; // distrust the codes: re-score everything
            } else if (iters <= kRegIters) {
                float lbs[kRegIters][4];
#pragma unroll
                for (int it = 0; it < kRegIters; ++it)
#pragma unroll
                    for (int e = 0; e < 4; ++e) lbs[it][e] = INFINITY;
                // one pass over all items; with dumps to copy, chunk by chunk
                const int span = chunk_len > 0 ? chunk_len : a.gstride;
                for (int cb = 0; cb < a.gstride; cb += span) {
                    if (chunk_len > 0) {
                        __syncthreads(); // the previous chunk has been read by everyone
                        chunk_base = cb;
                        gather_chunk(cb);
                        __syncthreads();
                    }
#pragma unroll
                    for (int it = 0; it < kRegIters; ++it) {
                        const int item = it * 512 + tid;
                        if (it < iters && item < items && it * 2048 >= cb && it * 2048 < cb + span) {
                            float ub4[4];
                            decode_item(item, ub4, lbs[it]);
                            ub_min = fminf(ub_min, fminf(fminf(ub4[0], ub4[1]), fminf(ub4[2], ub4[3])));
                        }
                    }
                }
                const float thr = block_min(ub_min) * 1.1893f * 1.0001f;
#pragma unroll
                for (int it = 0; it < kRegIters; ++it)
                    if (it < iters) list_candidates(it * 512 + tid, lbs[it], thr);
            } else { // budgets beyond the register window: decode twice (dump chunks are copied twice)
                const int span = chunk_len > 0 ? chunk_len : a.gstride;
                float thr = 0.f;
                for (int pass = 0; pass < 2; ++pass) {
                    for (int cb = 0; cb < a.gstride; cb += span) {
                        if (chunk_len > 0) {
                            __syncthreads(); // the previous chunk has been read by everyone
                            chunk_base = cb;
                            gather_chunk(cb);
                            __syncthreads();
                        }
                        const int it_hi = min(iters, (cb + span + 2047) / 2048); // the last span may be ragged
                        for (int it = cb / 2048; it < it_hi; ++it) {
                            const int item = it * 512 + tid;
                            if (item < items) {
                                float ub4[4], lb4[4];
                                decode_item(item, ub4, lb4);
                                if (pass == 0) ub_min = fminf(ub_min, fminf(fminf(ub4[0], ub4[1]), fminf(ub4[2], ub4[3])));
                                else list_candidates(item, lb4, thr);
                            }
                        }
                    }
                    if (pass == 0) thr = block_min(ub_min) * 1.1893f * 1.0001f;
                }
            }
            __syncthreads();
            const int ncand = cand_count;
            // exact double-precision scores of the candidates, one wave each
            double bv = INFINITY;
            int bi = 0x7fffffff;
            if (ncand == 1) {
                bi = cand_list[0]; // nothing to compare with: the screening already decided
                bv = 0.0;
            } else if (ncand <= kMaxCand) {
                for (int c = wave; c < ncand; c += NW) {
                    const int cs = cand_list[c];
                    if (bv == 0.0 && cs > bi) continue; // behind an exact zero nothing can win
                    const double v = __shfl(exact_score_bf16(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qs, G, sM, sL, lane,
                                                             COOP && s_active > 1 && cs == ins_slot), 0);
                    if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
                }
            } else {
                // Far more candidates than the list holds: scores underflowing en masse, or many
                // value rows of zero norm (a padded sequence).  Every wave takes its share of ALL
                // slots, 64 at a time in ascending order.  A row with ||v||_1 = 0 scores exactly 0
                // whatever its weight and needs no arithmetic (the side array says so; the row
                // written by this very step is not trusted to have arrived there and is re-scored
                // like any other); every other slot is re-scored exactly.  Scores are >= 0 and
                // ties go to the lower slot, so a wave is done at its first exact zero.
                for (int c0 = wave * 64; c0 < n && bv > 0.0; c0 += NW * 64) {
                    const int mine = c0 + lane;
                    bool zero = false;
                    if (mine < n && mine != ins_slot) zero = lu_u[(mine & ~15) + pos_of_slot(mine & 15)] == -INFINITY;
                    const unsigned long long zmask = __ballot(zero);
                    unsigned long long todo = __ballot(mine < n && !zero);
                    const int first_zero = zmask ? c0 + __ffsll((long long)zmask) - 1 : 0x7fffffff;
                    while (todo) {
                        const int cs = c0 + __ffsll((long long)todo) - 1;
                        todo &= todo - 1;
                        if (cs > first_zero) break; // cannot beat the zero in front of it
                        // (the score is complete in every fourth lane only: lane 0's goes to all,
                        // so that the exits below are taken by the whole wave)
                        const double v = __shfl(exact_score_bf16(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qs, G, sM, sL, lane,
                                                                 COOP && s_active > 1 && cs == ins_slot), 0);
                        if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
                        if (bv == 0.0) break;
                    }
                    if (zmask && (0.0 < bv || first_zero < bi)) { bv = 0.0; bi = first_zero; }
                }
            }
            if (lane == 0) { best_v[wave] = bv; best_i[wave] = bi; }
            __syncthreads();
            if (tid == 0) {
                double v = best_v[0];
                int i = best_i[0];
                for (int w = 1; w < NW; ++w)
                    if (best_v[w] < v || (best_v[w] == v && best_i[w] < i)) { v = best_v[w]; i = best_i[w]; }
                if (i < 0 || i >= N) i = 0; // non-finite scores: keep the slot in range
                a.pending[u] = i;
                if (a.evict_idx) a.evict_idx[u] = i;
            }
        }
        __syncthreads(); // the codes are dead from here on: their LDS may be reused below
    }

    // ---- output: normalise, round to bf16
    if (!COOP || s_active == 1) {
        stage_o();
        __syncthreads();
        for (int idx = tid; idx < G * D; idx += 512) {
            const int h = idx / D, d = idx % D;
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += sm_o[((size_t)w * G + h) * OPAD + d];
            a.out[((size_t)u * G + h) * D + d] = (uint16_t)f32_to_bf16_bits(acc / sL[h]);
        }
    } else { // the output was stored with the merge
        if (tid == 0) { // ready for the next step
            st_agent(&a.arrive[u], 0);
            st_agent(&a.dumped[u], dumps_ok ? 0 : kDumpsDistrusted);
        }
    }
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// O-merge area: one row of 128 (+4 padding) floats per wave and query head of the group
static size_t merge_bytes(int G) { return (size_t)8 * G * (128 + 4) * sizeof(float); }

static size_t code_bytes(int slots, int G)
{
    const size_t stride = ((size_t)slots + 63) / 64 * 64;
    return (size_t)G * stride + ((size_t)slots / kTile + 1) * G * sizeof(float);
}

// workgroups per unit: one when the units alone fill the chip, else enough to put a
// workgroup on (about) every compute unit, each with at least 256 slots
int unit_mfma_splits(int units, int N)
{
    if (units >= 192) return 1;
    int S = 256 / units;
    if (S > 8) S = 8;
    while (S > 1 && (N + S - 1) / S < 256) --S;
    return S < 1 ? 1 : S;
}

int unit_mfma_split_len(int N, int S)
{
    const int per = (N + S - 1) / S;
    return (per + 127) / 128 * 128;
}

size_t unit_mfma_lds_bytes(int N, int G, bool stash, int S)
{
    const size_t merge = merge_bytes(G);
    if (!stash) return merge;
    const size_t codes = code_bytes(unit_mfma_split_len(N, S), G);
    if (S == 1) return codes > merge ? codes : merge; // merge area aliases the codes
    return (codes + 255) / 256 * 256 + merge;
}

// One launch of one kernel instance.  The dynamic-LDS ceiling is a per-device function
// attribute: it is raised once per device and instance (attr_done, indexed by idx).
struct UnitLaunch {
    bool *attr_done;
    long long wgs;
    size_t lds;
    hipStream_t s;
    const UnitArgs *a;
    const GroupArgs *ga;
    bool masked, gather;
};

template <int STASH, bool COOP, bool GROUPED, bool MASKED, bool GATHER, bool MAXFREE>
static hipError_t launch_instance(const UnitLaunch &ul, int idx)
{
    auto kern = unit_mfma_kernel<true, STASH, COOP, GROUPED, MASKED, GATHER, MAXFREE>;
    if (!ul.attr_done[idx]) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kUnitLdsLimit);
        if (e != hipSuccess) return e;
        ul.attr_done[idx] = true;
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)ul.wgs), dim3(512), ul.lds, ul.s, *ul.a, *ul.ga);
    return hipGetLastError();
}

// The instances a (STASH, COOP, GROUPED) family really has: MASKED only where slots are
// scored, GATHER only where cooperating workgroups screen each other's codes.
template <int STASH, bool COOP, bool GROUPED>
static hipError_t launch_family(const UnitLaunch &ul, int idx)
{
    if constexpr (STASH == kStashLds) {
        if constexpr (COOP) {
            if (ul.gather)
                return ul.masked ? launch_instance<STASH, COOP, GROUPED, true, true, false>(ul, 24 + idx)
                                 : launch_instance<STASH, COOP, GROUPED, false, true, false>(ul, 16 + idx);
        }
        if (ul.masked) return launch_instance<STASH, COOP, GROUPED, true, false, false>(ul, 8 + idx);
    }
    return launch_instance<STASH, COOP, GROUPED, false, false, false>(ul, idx);
}

// everything of a step's kernel arguments that depends on the cache and the fill level only
static UnitArgs unit_args_of(const Plan &p, int n, int S)
{
    UnitArgs a;
    memset(&a, 0, sizeof(a));
    a.Kc = (uint16_t *)p.k_cache; a.Vc = (uint16_t *)p.v_cache;
    a.q_last = (uint16_t *)p.q_last;
    a.pending = p.pending;
    a.fin_m = p.fin_m; a.fin_l = p.fin_l; a.lu = p.lu;
    a.part_m = p.part_m; a.part_l = p.part_l; a.part_o = p.part_o;
    a.arrive = p.arrive; a.dumped = p.dumped;
    a.gcode = (uint8_t *)p.stash_w; a.gref = p.stash_m;
    a.n = n; a.N = p.N; a.G = p.G; a.ntiles = p.ntiles;
    a.S = S; a.split_len = unit_mfma_split_len(p.N, S);
    a.s_active = (n + a.split_len - 1) / a.split_len;
    a.code_stride = (a.split_len + 63) / 64 * 64;
    a.gstride = p.ntiles * kTile;
    const bool stash = !(p.flags & 1u);
    const size_t lds = unit_mfma_lds_bytes(p.N, p.G, stash, S);
    a.merge_off = (stash && S > 1) ? (int)(lds - merge_bytes(p.G)) : 0;
    a.chunk_len = 0;
    a.scale_log2 = 1.4426950408889634f / sqrtf(128.f);
    return a;
}

static_assert(sizeof(UnitArgs) <= kTableEntryMax && sizeof(UnitArgs) % 4 == 0, "entry travels as a kernel argument");
size_t unit_mfma_table_entry_bytes() { return sizeof(UnitArgs); }

void unit_mfma_table_entry(const Plan &p, void *dst)
{
    const UnitArgs a = unit_args_of(p, p.N, p.unit_S);
    memcpy(dst, &a, sizeof(a));
}

// `table` == nullptr: one cache, arguments by value.  Otherwise `n_caches` caches of p's
// geometry, all holding n - 1 (or N) rows, served by one grid; io holds the base pointers.
static hipError_t launch_unit(const Plan &p, const StepIo &io, int n, const void *table, int n_caches,
                              hipStream_t s)
{
    const bool stash = !(p.flags & 1u);
    // Workgroups per unit: the cache's own choice, made for it alone.  A group brings
    // n_caches times the units, so it needs fewer (never more: the cache's partial and
    // dump buffers are sized for its own choice) -- as long as the codes still fit LDS.
    int S = p.unit_S;
    if (table && S > 1) {
        int Sg = unit_mfma_splits((int)std::min<long long>((long long)p.units * n_caches, 1 << 20), p.N);
        while (Sg < S && unit_mfma_lds_bytes(p.N, p.G, stash, Sg) > kUnitLdsLimit) ++Sg;
        if (Sg < S) S = Sg;
    }
    UnitArgs a = unit_args_of(p, n, S);
    a.q = (const uint16_t *)io.q; a.k_new = (const uint16_t *)io.k_new; a.v_new = (const uint16_t *)io.v_new;
    a.out = (uint16_t *)io.out; a.evict_idx = io.evict_idx;
    GroupArgs ga;
    ga.table = (const UnitArgs *)table;
    ga.wgs_per_cache = p.units * a.s_active;
    ga.q_stride = (long long)p.units * p.G * 128;
    ga.kv_stride = (long long)p.units * 128;
    ga.ev_stride = p.units;
    size_t lds = unit_mfma_lds_bytes(p.N, p.G, stash, S);
    bool gather = false;
    if (stash && S > 1 && (p.N + a.split_len - 1) / a.split_len >= 3) {
        // From three workgroups per unit on, the deciding one copies the others' dumps into
        // LDS before screening them (with two, reading them in place is one batch of loads
        // as well, and measured 2 us faster on cfg2).  Room behind the own codes: 1 byte per
        // head and slot plus 4 bytes per head and 16 slots, in chunks of whole multiples of
        // 2048 positions -- as much as fits, at least 2048 (that much the merge area alone holds).
        const size_t per_pos4 = (size_t)p.G * 5; // bytes per 4 positions
        const size_t avail = kUnitLdsLimit - (size_t)a.merge_off;
        long long fit = (long long)(avail * 4 / per_pos4) / 2048 * 2048;
        const long long all = ((long long)p.ntiles * kTile + 2047) / 2048 * 2048;
        if (fit > all) fit = all;
        if (fit >= 2048) {
            gather = true;
            a.chunk_len = (int)fit;
            const size_t want = (size_t)a.merge_off + std::max((size_t)fit * per_pos4 / 4, merge_bytes(p.G));
            if (want > lds) lds = want;
        }
    }
    // With at most a few workgroups per compute unit, ask for more than half of the
    // CU's LDS so that no CU is handed two of them while another one idles.
    const long long wgs = (long long)ga.wgs_per_cache * n_caches;
    if (wgs <= 2 * 256 && lds < 81 * 1024) lds = 81 * 1024;
    if (wgs > 0x7fffffffll) return hipErrorInvalidValue;
    // the dynamic-LDS ceiling is a per-device function attribute: raise it once per device
    // and kernel instance (a benign race if two host threads get here together: both set it)
    constexpr int kMaxDevices = 64;
    static bool attr_done_all[kMaxDevices][34] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    bool *attr_done = attr_done_all[dev];
    // the mask only matters where slots are scored (an attention-only cache takes none), the
    // gathering only where cooperating workgroups screen codes
    const UnitLaunch ul = {attr_done, wgs, lds, s, &a, &ga, p.masked, gather};
    const bool coop = S > 1;
    if (p.max_free) { // attention only, one cache (the API layer admits nothing else)
        if (table || stash) return hipErrorInvalidValue;
        return coop ? launch_instance<kStashNone, true, false, false, false, true>(ul, 32)
                    : launch_instance<kStashNone, false, false, false, false, true>(ul, 33);
    }
    if (table) {
        if (stash) return coop ? launch_family<kStashLds, true, true>(ul, 4) : launch_family<kStashLds, false, true>(ul, 5);
        return coop ? launch_family<kStashNone, true, true>(ul, 6) : launch_family<kStashNone, false, true>(ul, 7);
    }
    if (stash) return coop ? launch_family<kStashLds, true, false>(ul, 0) : launch_family<kStashLds, false, false>(ul, 1);
    return coop ? launch_family<kStashNone, true, false>(ul, 2) : launch_family<kStashNone, false, false>(ul, 3);
}

hipError_t launch_unit_mfma(const Plan &p, const void *q, const void *k_new, const void *v_new, int n,
                            void *out, int32_t *evict_idx, hipStream_t s)
{
    const StepIo io = {q, k_new, v_new, out, evict_idx};
    return launch_unit(p, io, n, nullptr, 1, s);
}

hipError_t launch_unit_mfma_group(const Plan &p, const StepIo &io, int n, const void *table, int n_caches,
                                  hipStream_t s)
{
    return launch_unit(p, io, n, table, n_caches, s);
}

} // namespace lf
