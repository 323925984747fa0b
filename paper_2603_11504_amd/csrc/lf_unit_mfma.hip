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
//   evict    screen every slot with the codes (bounds within a known factor), re-score the
//            few that can still be the minimum exactly in double precision, argmin
//   output   normalise, round to bf16
//
// Keeping the per-slot by-products in LDS matters on this chip: even a few percent of HBM
// writes interleaved with the K/V read stream cost a quarter of the read bandwidth.
//
// Cooperation protocol for S > 1.  Nobody ever waits for anybody: each workgroup writes its
// partial (m, l, O) AND its codes (a dump of G bytes per slot, plus the per-tile references)
// through to the device-wide coherence point, waits for its own stores, and then bumps
// arrive[u] -- one counter, one bump per workgroup and step.  Whoever finds itself last has
// everything it needs already sitting at the coherence point: it fetches the partials and
// the other workgroups' dumps in one batch of loads (the dumps go straight into the LDS that
// held the O-merge area; a chunk at a time if they do not all fit), merges, stores the
// output, and decides the eviction from its own LDS codes plus the copies.  The last
// workgroup's own dump is wasted; that is the price of not having to wait for the others'.
#include <algorithm>
#include <cstring>

#include <atomic>
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
    int32_t *arrive;                   // [units], zero between steps
    uint8_t *gcode;                    // [units][G][gstride] dumped codes, absolute positions
    float *gref;                       // [units][ntiles][G] dumped references
    int n, N, G, ntiles;
    int S, s_active, split_len;        // split_len: slots per workgroup, a multiple of 256
    int code_stride, gstride;          // LDS / dump row strides in bytes
    int merge_off;                     // byte offset of the O-merge area in dynamic LDS (0 with one
                                       // workgroup per unit: the area then aliases the codes)
    int chunk_len;                     // positions of the other workgroups' dumps the deciding one holds in
                                       // LDS at a time (multiple of 2048; 0 with one workgroup per unit)
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
// (The pointers are cast to the global address space: on a generic pointer these become FLAT
// instructions, which count against the LDS counter as well, and every later wait for an LDS
// read would then wait for the trip to the coherence point too.)
template <typename T> __device__ __forceinline__ void st_agent(__attribute__((address_space(1))) T *p, T v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ void st_agent(T *p, T v)
{
    typedef __attribute__((address_space(1))) T *gptr;
    __hip_atomic_store((gptr)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ T ld_agent(__attribute__((address_space(1))) const T *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <typename T> __device__ __forceinline__ T ld_agent(const T *p)
{
    typedef __attribute__((address_space(1))) const T *gptr;
    return __hip_atomic_load((gptr)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int add_agent(int32_t *p, int v)
{
    typedef __attribute__((address_space(1))) int32_t *gptr;
    return __hip_atomic_fetch_add((gptr)p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// cache-policy operand of the loads that write LDS directly: the sc1 bit, i.e. device scope, what
// ld_agent's loads carry (the data comes from the coherence point, not from this XCD's L2)
constexpr int kAuxDeviceScope = 16;
typedef __attribute__((address_space(1))) const uint32_t *g_cu32p;
// all of this thread's device-scope stores have reached the coherence point
__device__ __forceinline__ void wait_stores() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Reductions of doubles for the exact re-scoring.  Inside a row of 16 lanes they go through DPP
// (a few cycles a level); only the two levels across rows take the cross-lane permute, whose
// latency is an order of magnitude more and stands in the serial tail of the kernel.
template <int CTRL> __device__ __forceinline__ double dpp_f64(double x)
{
    const long long b = __double_as_longlong(x);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)b, CTRL, 0xf, 0xf, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double rows_sum_f64(double x) // over the four rows: same position in each
{
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}
__device__ __forceinline__ double wave_sum_f64(double x)
{
    x += dpp_f64<0x128>(x); // row_ror:8
    x += dpp_f64<0x124>(x); // row_ror:4
    x += dpp_f64<0x122>(x); // row_ror:2
    x += dpp_f64<0x121>(x); // row_ror:1
    return rows_sum_f64(x);
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

// One cache row pair as the exact re-scoring wants it: lane (h = lane >> 2, part = lane & 3)
// holds K channels 32 part .. 32 part + 31 and two V channels.  Loading and scoring are
// separate steps so that a wave can have its candidate's rows on their way while it does
// something else.
struct RowRegs {
    uint32_t vv;
    u32x4 kk[4];
};
//   coherent: read the row with device-scope loads (it was written during this launch by
//   another workgroup)
__device__ __forceinline__ void load_row(RowRegs &rr, g_cu16p krow, g_cu16p vrow, int lane, bool coherent)
{
    const int part = lane & 3;
    rr.vv = coherent ? ld_agent((g_cu32p)vrow + lane) : *(g_cu32p)(vrow + 2 * lane);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        if (coherent) {
            const g_cu32p kp = (g_cu32p)(krow + 32 * part + 8 * c);
            rr.kk[c] = u32x4{ld_agent(kp), ld_agent(kp + 1), ld_agent(kp + 2), ld_agent(kp + 3)};
        } else {
            rr.kk[c] = *(g_cu32x4p)(krow + 32 * part + 8 * c);
        }
    }
}

// Exact LongFlowScore of one slot in double precision (eq. 6 with the group's heads
// summed), computed by one wave: 4 lanes per head, 32 channels per lane.
//   qs: the step's query in LDS [16][128]; sM: softmax reference per head (log2 domain);
//   sL: denominator per head.  The result is complete in every fourth lane.
__device__ __forceinline__ double score_row(const RowRegs &rr, const uint16_t (*qs)[128], int G, const float *sM, const float *sL, int lane)
{
    const int h = lane >> 2, part = lane & 3;
    // ||v||_1: two channels per lane, summed over the wave
    double l1 = fabs((double)bf16_lo(rr.vv)) + fabs((double)bf16_hi(rr.vv));
    l1 = wave_sum_f64(l1);
    // q_h . k over this lane's 32 channels
    double dot = 0.0;
    if (h < G) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const u32x4 kk = rr.kk[c];
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
    dot += dpp_f64<0xB1>(dot); // quad_perm [1,0,3,2]: the neighbour in the pair
    dot += dpp_f64<0x4E>(dot); // quad_perm [2,3,0,1]: the other pair of the four lanes of a head
    double term = 0.0;
    if (h < G && part == 0) {
        const double scale_log2 = 1.4426950408889634074 / 11.313708498984760390; // log2(e) / sqrt(128)
        const double d = dot * scale_log2 - (double)sM[h];
        const double nint = rint(d);
        term = ldexp(exp2_frac_f64(d - nint), (int)nint) / (double)sL[h];
    }
    // the heads' terms sit in every fourth lane (zeros between them): rotations by 4 and 8 add up
    // the four heads of a row in each of those lanes, then the rows
    term += dpp_f64<0x124>(term); // row_ror:4
    term += dpp_f64<0x128>(term); // row_ror:8
    return rows_sum_f64(term) * l1;
}

__device__ __forceinline__ double exact_score_bf16(g_cu16p krow, g_cu16p vrow, const uint16_t (*qs)[128], int G,
                                   const float *sM, const float *sL, int lane, bool coherent)
{
    RowRegs rr;
    load_row(rr, krow, vrow, lane, coherent);
    return score_row(rr, qs, G, sM, sL, lane);
}

// Explicit-mask mode: the lowest invalid slot of the unit (NaN in the side array), not
// counting the slot this step has just filled (its entry may still read stale here).
// All 512 threads call; true if there is one, then it is in red[0].
__device__ bool fill_lowest_hole(g_cf32p lu_u, int npos, int N, int ins_slot, int *red, int tid, int lane,
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

// Screening.  A code c stands for 2^(kCodeBias - c/4).
// For a code that sits at no clamp the true term t and its decoded value d obey
//   d 2^(-1/8) <= t <= d 2^(1/8)
// (rounding of the code: half a step of 1/4 either way).  Sums over the heads inherit the
// bounds, so slot i can hold the smallest true sum only if  sum_i <= min_j sum_j * 2^(1/4);
// the last factor below covers the fp32 rounding of the sums and of the code's argument.
constexpr float kScreenWindow = 1.189208f * 1.0002f;

// COOP: several workgroups may share a unit (s_active can exceed 1)
// MAXFREE: softmax without a running reference (Alg. 1 as printed), for A/B measurement; the codes are then
// relative to the fixed reference 0 and clamp (one-sided bounds, still rigorous) once ||v||_1 2^t leaves
// [2^-48, 2^16]
// (Every lambda below is marked always_inline: a real call would make the compiler keep the
// kernel's arguments, which the lambdas capture by reference, in private memory, and a load from
// there waits for every outstanding store -- which serialises the device-scope stores.)
template <bool HILO, int STASH, bool COOP, bool GROUPED, bool MASKED, bool MAXFREE = false>
__global__ __launch_bounds__(512, 1) void unit_mfma_kernel(const UnitArgs a_in, const GroupArgs ga)
{
    UnitArgs a = a_in;
    // (every argument the start of the kernel reads is asked for here, in one batch of scalar loads:
    // left alone, the compiler fetches them in two, the second behind the first's wait)
    asm volatile("" ::"s"(a.Kc), "s"(a.pending), "s"(a.lu), "s"(a.n), "s"(a.split_len), "s"(a.code_stride), "s"(a.merge_off),
                 "s"(a.scale_log2));
    int blk = blockIdx.x;
    if (GROUPED) {
        // which cache this workgroup serves; the geometry and the step's scalars are common
        const int ci = blk / ga.wgs_per_cache;
        blk -= ci * ga.wgs_per_cache;
        const UnitArgs *t = ga.table + ci;
        a.Kc = (t->Kc); a.Vc = (t->Vc); a.q_last = (t->q_last); a.pending = (t->pending);
        a.fin_m = (t->fin_m); a.fin_l = (t->fin_l); a.lu = (t->lu);
        a.part_m = (t->part_m); a.part_l = (t->part_l); a.part_o = (t->part_o);
        a.arrive = (t->arrive); a.gcode = (t->gcode); a.gref = (t->gref);
        a.q += ci * ga.q_stride;
        a.out += ci * ga.q_stride;
        if (a.k_new) a.k_new += ci * ga.kv_stride;
        if (a.v_new) a.v_new += ci * ga.kv_stride;
        if (a.evict_idx) a.evict_idx += ci * ga.ev_stride;
    }
    constexpr int D = 128, NW = 8, OPAD = D + 4;
    extern __shared__ __align__(16) unsigned char smem[];
    // dynamic LDS: [codes G*code_stride][refs (split_len/16)*G floats] ... [O-merge area
    // [NW][G][OPAD] floats at merge_off].  With one workgroup per unit and codes too large to
    // leave room, merge_off is 0: the area then aliases the codes and is used after them.
    uint8_t *ls_code = smem;
    float *ls_ref = (float *)(smem + (size_t)a.G * a.code_stride);
    float *sm_o = (float *)(smem + a.merge_off);
    __shared__ float sm_m[NW][16], sm_l[NW][16], sM[16], sL[16];
    __shared__ float sLg[16]; // kCodeBias - reference - log2 denominator per head: what turns a tile's reference into the log2 factor of its codes
    __shared__ float sW[8][16]; // weights of the S partials under the unit-wide reference
    __shared__ float red_f[NW];
    __shared__ double best_v[NW];
    __shared__ int best_i[NW];
    __shared__ __align__(16) uint16_t qs[16][D]; // the query, for the exact re-scoring
    __shared__ int cand_list[kMaxCand];
    __shared__ int cand_count, s_flag;
    __shared__ int red_i[NW + 1];

    const int n = a.n, N = a.N, G = a.G, s_active = COOP ? a.s_active : 1;
    const int u = blk / s_active, sp = blk % s_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    const int start = sp * a.split_len;
    const int end = min(start + a.split_len, n);
    // (global address space by type, see lf_mfma_stream.h: no access below may turn into a FLAT
    // instruction, whose completion can only be awaited together with the LDS counter)
    typedef __attribute__((address_space(1))) int32_t *g_i32p;
    const g_u16p Ku = (g_u16p)a.Kc + (size_t)u * N * D;
    const g_u16p Vu = (g_u16p)a.Vc + (size_t)u * N * D;
    const g_cu16p qu = (g_cu16p)a.q + (size_t)u * G * D;
    const g_f32p lu_u = (g_f32p)a.lu + (size_t)u * a.ntiles * kTile;
    const g_cu16p k_new = (g_cu16p)a.k_new, v_new = (g_cu16p)a.v_new;
    const g_u16p out_g = (g_u16p)a.out, q_last = (g_u16p)a.q_last;
    const g_i32p pending = (g_i32p)a.pending, evict_idx = (g_i32p)a.evict_idx;
    const g_f32p fin_m = (g_f32p)a.fin_m, fin_l = (g_f32p)a.fin_l;
    const bool evicting = (STASH == kStashLds) && n == N;
    const bool coop = COOP && s_active > 1;
    // the O-merge area has LDS of its own (it does not alias live codes): the output can be
    // staged before the eviction decision and stored while candidates' rows are on their way
    const bool o_separate = STASH != kStashLds || a.merge_off != 0;

    // ---- insert (Fig. 2 left): done by the wave that will stream that tile, so that its own
    // later loads of the row are ordered behind the stores.  The row is written through to
    // the device-wide coherence point: with several workgroups per unit, the one that ends
    // up re-scoring candidates may sit on another XCD and must not see the old row.
    // Everything the kernel needs from memory before it can stream is requested in one go, and nothing
    // is used before all of it has been asked for: the pending slot, the query (once for the copies
    // below, once as the matrix operand), the wave's first three tiles.  One trip to memory at the start
    // of the kernel, where a load followed by its use, three times over, had cost three.  (No loop may
    // stand between a request and its use: the compiler drains every outstanding load in front of one.)
    // (the unit index goes through a vector register the compiler cannot see through: a load it knows to
    // be uniform it moves to a scalar register at once, which waits for it on the spot)
    int u_vec = u;
    asm volatile("" : "+v"(u_vec));
    const int ins_slot = (STASH != kStashNone) ? pending[u_vec] : -1;
    // the query, 4 elements a thread: G * D <= 2048 = 512 x 4
    const bool q_mine = 4 * tid < G * D;
    u32x2 q4 = {0u, 0u};
    if (q_mine) q4 = *(g_cu32x2p)(qu + 4 * tid);
    // the new token's row, by every wave: which one inserts it is known only when the pending slot is
    uint32_t new_k = 0u, new_v = 0u;
    u32x4 new_vv = {0u, 0u, 0u, 0u};
    if (STASH != kStashNone && k_new && v_new) {
        new_k = *((g_cu32p)(k_new + (size_t)u * D) + lane);
        new_v = *((g_cu32p)(v_new + (size_t)u * D) + lane);
        new_vv = *(g_cu32x4p)(v_new + (size_t)u * D + 8 * r);
    }

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
    TileRegs ta, tb, tc;
    const bool requested = st.request_first_tiles(wave, ta, tb, tc);

    // Copies of the query -- LDS for the exact re-scoring, device memory for a later
    // longflow_scores() -- made at the start: their latency hides behind the streaming instead of
    // standing in the serial tail of the kernel.
    if (q_mine) {
        if (STASH == kStashLds) *(u32x2 *)(&qs[0][0] + 4 * tid) = q4;
        if (sp == 0) *(g_u32x2p)(q_last + (size_t)u * G * D + 4 * tid) = q4;
    }

    if (STASH != kStashNone) {
        const int slot = ins_slot;
        if (slot >= start && slot < start + a.split_len && slot < N && (((slot - start) / kTile) % NW) == wave) {
            st_agent((g_u32p)(Ku + (size_t)slot * D) + lane, new_k);
            st_agent((g_u32p)(Vu + (size_t)slot * D) + lane, new_v);
            // every 16-lane row sums |v_new| redundantly; lane 0 stores the log2 norm
            const u32x4 vv = new_vv;
            float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                       fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
            a1 = row16_sum(a1);
            if (lane == 0) lu_u[(slot & ~15) + pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            // a tile requested above may hold the row as it was: ask for it again, behind the stores
            if (requested) {
                const int ti = (slot - start) / kTile;
                if (ti == wave) st.template load_tile<false>(ta, ti);
                else if (ti == wave + NW) st.template load_tile<false>(tb, ti);
                else if (ti == wave + 2 * NW) st.template load_tile<false>(tc, ti);
            }
        }
    }

    st.run(wave, ta, tb, tc, requested);

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
        sLg[tid] = kCodeBias - M - __builtin_amdgcn_logf(Ls);
    }
    __syncthreads();

    // O of the 8 waves -> LDS, each under this workgroup's reference
    auto stage_o = [&]() __attribute__((always_inline)) {
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
    // normalised output of a unit served by this workgroup alone
    auto store_out = [&]() __attribute__((always_inline)) {
        for (int idx = tid; idx < G * D; idx += 512) {
            const int h = idx / D, d = idx % D;
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += sm_o[((size_t)w * G + h) * OPAD + d];
            out_g[((size_t)u * G + h) * D + d] = (uint16_t)f32_to_bf16_bits(acc / sL[h]);
        }
    };

    // the same for a unit shared by several workgroups: the S partial outputs come from the
    // coherence point (requested with the last arriver's first batch of loads, used here) and
    // are weighted under the unit-wide reference
    constexpr int kOutPer = (kMaxGroup * D + 511) / 512;
    float po[kOutPer][8];
    auto request_partial_outputs = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kOutPer; ++k) {
            const int idx = tid + 512 * k;
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2)
                po[k][s2] = (idx < G * D && s2 < s_active)
                                ? ld_agent(&a.part_o[((size_t)u * a.S + s2) * G * D + idx]) : 0.f;
        }
    };
    auto merge_out = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kOutPer; ++k) {
            const int idx = tid + 512 * k;
            if (idx < G * D) {
                const int h = idx / D;
                float acc = 0.f;
#pragma unroll
                for (int s2 = 0; s2 < 8; ++s2) acc += sW[s2][h] * po[k][s2];
                out_g[(size_t)u * G * D + idx] = (uint16_t)f32_to_bf16_bits(acc / sL[h]);
            }
        }
    };

    // the other workgroups' codes in LDS, a chunk of positions at a time (COOP only): where the
    // O-merge area was, dead once the partial has been published
    const int own_hi = min(start + a.split_len, a.gstride);
    const int chunk_len = coop ? a.chunk_len : 0;
    uint8_t *rem_code = smem + a.merge_off;
    float *rem_ref = (float *)(rem_code + (size_t)G * chunk_len);
    // Copy the dumps of positions [cb, cb + chunk_len) into LDS, references as dumped.  The own range
    // inside the chunk, [lo, hi) relative to cb, is skipped for the codes (they are in LDS already);
    // the references, a quarter of the volume, are copied whole.  The loads write LDS directly
    // (`global_load_lds_dword`, device scope): a wave instruction moves 256 consecutive bytes, no
    // register holds anything, so ONE short loop has every load of the chunk in flight at once --
    // every device-scope load is a trip to the coherence point and a batch of them costs about one --
    // and the code is a few dozen instructions where a register-staged batch took over a thousand
    // (this runs once per launch, in the serial tail of the deciding workgroup: its instruction count
    // is its cost).  Ranges are whole runs: split_len and chunk_len are multiples of 256.
    // gather_wait() before the barrier behind which the chunk is read.
    typedef __attribute__((address_space(3))) void *lds_vp;
    typedef __attribute__((address_space(1))) const uint8_t *g_cu8p;
    auto gather_chunk = [&](int cb) __attribute__((always_inline)) {
        const int lo = min(max(start - cb, 0), chunk_len), hi = min(max(start + a.split_len - cb, 0), chunk_len);
        const int skip = hi - lo;
        const int runs_per_h = (chunk_len - skip) / 256;
        const int last = a.gstride - 4; // last word of a dump row: positions beyond it are dead
        for (int h = 0; h < G; ++h) {
            const g_cu8p row = (g_cu8p)a.gcode + ((size_t)u * G + h) * a.gstride;
            for (int j = wave; j < runs_per_h; j += NW) {
                int o = 256 * j;
                if (o >= lo) o += skip;
                __builtin_amdgcn_global_load_lds((g_cu32p)(row + min(cb + o + 4 * lane, last)),
                                                 (lds_vp)(rem_code + (size_t)h * chunk_len + o), 4, 0, kAuxDeviceScope);
            }
        }
        const int have = (a.ntiles - cb / kTile) * G; // references from cb to the end of the unit
        const g_cf32p src = (g_cf32p)a.gref + ((size_t)u * a.ntiles + cb / kTile) * G;
        for (int j = wave; 64 * j < (chunk_len / kTile) * G; j += NW)
            __builtin_amdgcn_global_load_lds(src + min(64 * j + lane, have - 1), (lds_vp)(rem_ref + 64 * j), 4, 0, kAuxDeviceScope);
    };
    auto gather_wait = [&]() __attribute__((always_inline)) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    // A code c of head h in a tile whose reference the streaming left at `ref` stands for the term
    // 2^(ref + sLg[h] - c/4) of the score: one conversion, one multiply-add and one exponential per
    // code, no table (a 256-entry table in LDS cost more in bank conflicts than the exponentials do).
    auto code_term = [&](uint32_t c4, int e, float lf) __attribute__((always_inline)) {
        return fast_exp2(fmaf((float)((c4 >> (8 * e)) & 255u), -0.25f, lf));
    };

    if (coop) {
        // ---- publish this workgroup's partial (m, l, O), and its codes if slots will be scored
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
        if (evicting) {
            const int len = (end - start + kTile - 1) / kTile * kTile; // whole tiles
            uint8_t *gc = a.gcode + (size_t)u * G * a.gstride + start;
            const int gstride = a.gstride, cstride = a.code_stride;
            for (int h = 0; h < G; ++h)
                for (int j = tid; j < len / 8; j += 512)
                    st_agent((unsigned long long *)(gc + (size_t)h * gstride + 8 * j),
                             *(const unsigned long long *)(ls_code + (size_t)h * cstride + 8 * j));
            float *gr = a.gref + ((size_t)u * a.ntiles + start / kTile) * G;
            for (int i = tid; i < (len / kTile) * G; i += 512) st_agent(gr + i, ls_ref[i]);
        }
        wait_stores();
        __syncthreads(); // every thread's stores are visible device-wide before the arrival counts
        if (tid == 0)
            s_flag = (add_agent(&a.arrive[u], 1) == s_active - 1);
        __syncthreads();
        if (!s_flag) return;
        // ---- last arriver: everything of the unit is at the coherence point.  One batch of
        // device-scope loads fetches the S softmax states and the first chunk of the others'
        // codes, and the partial outputs, which are not used before the decision is made.
        float pm[8], pl[8];
        request_partial_outputs();
        if (tid < 16) {
#pragma unroll
            for (int s2 = 0; s2 < 8; ++s2) {
                pm[s2] = -INFINITY;
                pl[s2] = 0.f;
                if (s2 < s_active) {
                    pm[s2] = ld_agent(&a.part_m[((size_t)u * a.S + s2) * 16 + tid]);
                    pl[s2] = ld_agent(&a.part_l[((size_t)u * a.S + s2) * 16 + tid]);
                }
            }
        }
        if (evicting) gather_chunk(0);
        if (tid < 16) {
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
            sLg[tid] = kCodeBias - M - __builtin_amdgcn_logf(Ls);
        }
        gather_wait();
        __syncthreads();
    } else if (o_separate && STASH == kStashLds) {
        stage_o(); // read back below, after the barriers of the decision
    }
    if (tid < G) {
        fin_m[(size_t)u * G + tid] = sM[tid];
        fin_l[(size_t)u * G + tid] = sL[tid];
    }

    // ---- eviction decision (Sec. 3.2 last paragraph; Alg. 1 post-processing)
    bool out_stored = false;
    if (STASH == kStashLds) {
        if (n < N) {
            if (tid == 0) {
                pending[u] = n;
                if (evict_idx) evict_idx[u] = n;
            }
        } else if (MASKED && fill_lowest_hole(lu_u, a.gstride, N, ins_slot, red_i, tid, lane, wave)) {
            // an invalid slot exists: it takes the next token, nothing is evicted
            if (tid == 0) {
                pending[u] = red_i[0];
                if (evict_idx) evict_idx[u] = red_i[0];
            }
        } else {
            int chunk_base = 0;
            // Decode every (head, slot) code once.  Each thread keeps the sums of its slots in
            // registers, the block finds the smallest, and a slot can be the true minimum only
            // if its sum lies within kScreenWindow of it.  A code at a clamp has no bound on one
            // side (0: no upper bound, 255: no lower bound) and sends its item through the
            // two-sided sums.
            const int items = 4 * ((n + kTile - 1) / kTile); // 4 positions each, whole tiles
            constexpr int kRegIters = 8; // 512 threads x 4 positions x 8 = 16384 slots held in registers
            const int iters = (items + 511) / 512;
            // where an item's codes and factors live, as byte offsets into dynamic LDS
            const int ref_off = G * a.code_stride, rem_off = a.merge_off, rem_ref_off = a.merge_off + G * chunk_len;
            auto item_source = [&](int item, int &cp, int &fp, int &cstride) __attribute__((always_inline)) {
                const int tile = item >> 2;
                cp = 4 * item;
                fp = ref_off + 4 * tile * G;
                cstride = a.code_stride;
                if (COOP) {
                    if (4 * item >= start && 4 * item < own_hi) {
                        cp = 4 * item - start;
                        fp = ref_off + 4 * (tile - start / kTile) * G;
                    } else { // another workgroup's: in the chunk that is in LDS right now
                        const int rp = 4 * item - chunk_base;
                        cp = rem_off + rp;
                        fp = rem_ref_off + 4 * (rp / kTile) * G;
                        cstride = chunk_len;
                    }
                }
            };
            auto decode_item = [&](int item, float *ub4, float *lb4) __attribute__((always_inline)) {
                int cpo, fpo, cstride;
                item_source(item, cpo, fpo, cstride);
                const uint8_t *cp = smem + cpo;
                const float *fp = (const float *)(smem + fpo);
                // Common case first: no code of the item sits at a clamp (0x00 or 0xff), so upper
                // and lower bound share one sum.  The byte tests are the usual word-at-a-time ones.
                uint32_t clamped = 0u;
                float s4[4] = {0.f, 0.f, 0.f, 0.f};
                for (int h = 0; h < G; ++h) {
                    const uint32_t c4 = *(const uint32_t *)(cp + (size_t)h * cstride);
                    const float lf = fp[h] + sLg[h];
                    clamped |= ((c4 - 0x01010101u) & ~c4) | ((~c4 - 0x01010101u) & c4);
#pragma unroll
                    for (int e = 0; e < 4; ++e) s4[e] += code_term(c4, e, lf);
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = s4[e];
                if (clamped & 0x80808080u) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = 0.f;
                    for (int h = 0; h < G; ++h) {
                        const uint32_t c4 = *(const uint32_t *)(cp + (size_t)h * cstride);
                        const float lf = fp[h] + sLg[h];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t c = (c4 >> (8 * e)) & 255u;
                            const float d = code_term(c4, e, lf);
                            ub4[e] += (c == 0u) ? INFINITY : d;
                            lb4[e] += (c == 255u) ? 0.f : d;
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int slot = ((4 * item) & ~15) + slot_of_pos((4 * item + e) & 15);
                    if (slot >= n) { ub4[e] = INFINITY; lb4[e] = INFINITY; }
                }
            };
            auto list_candidates = [&](int item, const float *lb4, float thr) __attribute__((always_inline)) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (lb4[e] <= thr) {
                        const int k = atomicAdd(&cand_count, 1);
                        if (k < kMaxCand) cand_list[k] = ((4 * item) & ~15) + slot_of_pos((4 * item + e) & 15);
                    }
                }
            };
            auto block_min = [&](float x) __attribute__((always_inline)) {
#pragma unroll
                for (int off = 32; off > 0; off >>= 1) x = fminf(x, __shfl_xor(x, off));
                if (lane == 0) red_f[wave] = x;
                __syncthreads();
                x = red_f[0];
#pragma unroll
                for (int w = 1; w < NW; ++w) x = fminf(x, red_f[w]);
                return x;
            };
            // chunk cb of the others' dumps into LDS, unless it is the one that is there (chunk 0
            // came with the partials)
            auto next_chunk = [&](int cb) __attribute__((always_inline)) {
                if (chunk_len == 0 || cb == chunk_base) return;
                __syncthreads(); // the previous chunk has been read by everyone
                chunk_base = cb;
                gather_chunk(cb);
                gather_wait();
                __syncthreads();
            };
            float ub_min = INFINITY;
            const int span = chunk_len > 0 ? chunk_len : a.gstride;
            if (iters <= kRegIters) {
                float lbs[kRegIters][4];
#pragma unroll
                for (int it = 0; it < kRegIters; ++it)
#pragma unroll
                    for (int e = 0; e < 4; ++e) lbs[it][e] = INFINITY;
                // One pass over all items; with dumps to copy, chunk by chunk.  The loop over the
                // heads is the outer one and the thread's items (a compile-time count NI >= iters)
                // are read unconditionally -- a dead item reads item 0's words and drops them -- so
                // that the LDS reads of one head are all in flight before the first is used.
                auto pass = [&](auto ni_tag, int cb) __attribute__((always_inline)) {
                    constexpr int NI = decltype(ni_tag)::value;
                    int cp[NI], fp[NI], cstr[NI]; // byte offsets into dynamic LDS
                    bool live[NI];
                    uint32_t clamped[NI];
                    float s4[NI][4];
#pragma unroll
                    for (int it = 0; it < NI; ++it) {
                        const int item = it * 512 + tid;
                        live[it] = item < items && it * 2048 >= cb && it * 2048 < cb + span;
                        item_source(live[it] ? item : (COOP ? start / 4 : 0), cp[it], fp[it], cstr[it]);
                        clamped[it] = 0u;
#pragma unroll
                        for (int e = 0; e < 4; ++e) s4[it][e] = 0.f;
                    }
                    for (int h = 0; h < G; ++h) {
                        uint32_t c4[NI];
                        float f[NI];
                        const float lgh = sLg[h];
#pragma unroll
                        for (int it = 0; it < NI; ++it) {
                            c4[it] = *(const uint32_t *)(smem + cp[it]);
                            f[it] = *(const float *)(smem + fp[it]);
                            cp[it] += cstr[it];
                            fp[it] += 4;
                        }
#pragma unroll
                        for (int it = 0; it < NI; ++it) {
                            f[it] += lgh;
                            clamped[it] |= ((c4[it] - 0x01010101u) & ~c4[it]) | ((~c4[it] - 0x01010101u) & c4[it]);
#pragma unroll
                            for (int e = 0; e < 4; ++e) s4[it][e] += code_term(c4[it], e, f[it]);
                        }
                    }
                    uint32_t redo = 0u; // items with a code at a clamp
#pragma unroll
                    for (int it = 0; it < NI; ++it) {
                        if (live[it]) {
                            if (clamped[it] & 0x80808080u) {
                                redo |= 1u << it;
                            } else {
                                // (a position past the last slot carries the clamp code 255 -- the streaming
                                // writes it so -- and has sent its item down the other branch)
#pragma unroll
                                for (int e = 0; e < 4; ++e) lbs[it][e] = s4[it][e];
                                ub_min = fminf(ub_min, fminf(fminf(s4[it][0], s4[it][1]), fminf(s4[it][2], s4[it][3])));
                            }
                        }
                    }
                    // The rare items take the two-sided sums in a loop of their own, so that the kernel
                    // holds that code once per pass and not once per item (the tail of a workgroup runs
                    // once, out of a cold instruction cache: its size is its cost).
#pragma nounroll
                    while (redo) {
                        const int it = __ffs(redo) - 1;
                        redo &= redo - 1u;
                        float ub4[4], lb4[4];
                        decode_item(it * 512 + tid, ub4, lb4);
#pragma unroll
                        for (int j = 0; j < NI; ++j) { // selects, not an indexed store: lbs stays in registers
                            const bool hit = j == it;
#pragma unroll
                            for (int e = 0; e < 4; ++e) lbs[j][e] = hit ? lb4[e] : lbs[j][e];
                        }
                        ub_min = fminf(ub_min, fminf(fminf(ub4[0], ub4[1]), fminf(ub4[2], ub4[3])));
                    }
                };
                // (the item count is dispatched on outside the loop over chunks: inside it, the compiler
                // hoists every instantiation's invariants in front of the loop and all of them are paid)
                auto all_chunks = [&](auto ni_tag) __attribute__((always_inline)) {
                    for (int cb = 0; cb < a.gstride; cb += span) {
                        next_chunk(cb);
                        pass(ni_tag, cb);
                    }
                };
                if (iters <= 1) all_chunks(std::integral_constant<int, 1>{});
                else if (iters <= 2) all_chunks(std::integral_constant<int, 2>{});
                else if (iters <= 4) all_chunks(std::integral_constant<int, 4>{});
                else all_chunks(std::integral_constant<int, kRegIters>{});
                const float thr = block_min(ub_min) * kScreenWindow;
                // one bit per position of the thread that may hold the minimum; the (few) set bits are
                // listed by one loop, so the kernel holds the listing code once and not per register
                uint32_t hits = 0u;
#pragma unroll
                for (int it = 0; it < kRegIters; ++it)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (it < iters && lbs[it][e] <= thr) hits |= 1u << (4 * it + e);
#pragma nounroll
                while (hits) {
                    const int b = __ffs(hits) - 1;
                    hits &= hits - 1u;
                    const int pos = 4 * ((b >> 2) * 512 + tid) + (b & 3);
                    const int k = atomicAdd(&cand_count, 1);
                    if (k < kMaxCand) cand_list[k] = (pos & ~15) + slot_of_pos(pos & 15);
                }
            } else { // budgets beyond the register window: decode twice (dump chunks are copied twice)
                float thr = 0.f;
                for (int pass = 0; pass < 2; ++pass) {
                    for (int cb = 0; cb < a.gstride; cb += span) {
                        next_chunk(cb);
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
                    if (pass == 0) thr = block_min(ub_min) * kScreenWindow;
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
                // A wave takes its candidates two at a time: both rows are requested, then (first round
                // only) the output is stored if this workgroup owes it and has it staged, then the rows
                // are used -- 16 candidates cost the workgroup one trip to memory, and the output's
                // stores hide behind the first.
                auto take = [&](double v, int cs) __attribute__((always_inline)) {
                    if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
                };
                for (int cb = 0; cb < ncand; cb += 2 * NW) { // uniform over the workgroup
                    RowRegs r0, r1;
                    const int c0 = cb + wave, c1 = cb + wave + NW;
                    // behind an exact zero nothing can win: such candidates are not even fetched
                    const bool use0 = c0 < ncand && !(bv == 0.0 && cand_list[c0] > bi);
                    const bool use1 = c1 < ncand && !(bv == 0.0 && cand_list[c1] > bi);
                    if (use0) {
                        const int cs = cand_list[c0];
                        load_row(r0, Ku + (size_t)cs * D, Vu + (size_t)cs * D, lane, coop && cs == ins_slot);
                    }
                    if (use1) {
                        const int cs = cand_list[c1];
                        load_row(r1, Ku + (size_t)cs * D, Vu + (size_t)cs * D, lane, coop && cs == ins_slot);
                    }
                    if (cb == 0) {
                        if (coop) { merge_out(); out_stored = true; }
                        else if (o_separate) { store_out(); out_stored = true; }
                    }
                    // (both rows through one copy of the scoring code: the second moves into the first's registers)
                    bool use = use0;
                    int c = c0;
#pragma nounroll
                    for (int k = 0; k < 2; ++k) {
                        if (use) take(__shfl(score_row(r0, qs, G, sM, sL, lane), 0), cand_list[c]);
                        r0 = r1;
                        use = use1;
                        c = c1;
                    }
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
                                                                 coop && cs == ins_slot), 0);
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
                pending[u] = i;
                if (evict_idx) evict_idx[u] = i;
            }
        }
    }

    // ---- output: normalise, round to bf16
    if (!out_stored && coop) {
        merge_out();
    } else if (!out_stored) {
        if (!(o_separate && STASH == kStashLds)) {
            __syncthreads(); // the codes are dead from here on: their LDS is reused
            stage_o();
        }
        __syncthreads();
        store_out();
    }
    if (coop && tid == 0) st_agent(&a.arrive[u], 0); // ready for the next step
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
    return (per + 255) / 256 * 256; // whole rounds of the 8 waves' tiles, and whole 256-byte runs of the code exchange
}

// How a workgroup's dynamic LDS is laid out for S workgroups per unit.
struct UnitLds {
    size_t merge_off; // where the O-merge area starts (0: it aliases the codes)
    int chunk_len;    // S > 1: positions of the other workgroups' dumps held at a time
    size_t bytes;
};
static UnitLds unit_lds(int N, int G, bool stash, int S)
{
    UnitLds l = {0, 0, merge_bytes(G)};
    if (!stash) return l;
    const size_t codes = (code_bytes(unit_mfma_split_len(N, S), G) + 255) / 256 * 256;
    if (S == 1) {
        // the merge area gets LDS of its own where there is room for it (the output is then
        // staged early and stored while candidates are re-scored), else it aliases the codes
        if (codes + merge_bytes(G) <= kUnitLdsLimit) { l.merge_off = codes; l.bytes = codes + merge_bytes(G); }
        else l.bytes = std::max(codes, merge_bytes(G));
        return l;
    }
    // Behind the own codes: first the O-merge area, then (in the deciding workgroup) the others'
    // dumps, 1 byte per head and slot plus 4 bytes per head and 16 slots, in chunks of whole
    // multiples of 2048 positions -- as much as fits, at least 2048 (that much the merge area
    // alone holds), at most all of them.
    l.merge_off = codes;
    const size_t per_pos4 = (size_t)G * 5; // bytes per 4 positions
    constexpr size_t kRefSlack = 256;      // the references arrive in runs of 64: the last one may overshoot
    const size_t avail = kUnitLdsLimit > codes + kRefSlack ? kUnitLdsLimit - codes - kRefSlack : 0;
    long long fit = (long long)(avail * 4 / per_pos4) / 2048 * 2048;
    const long long all = (((long long)N + kTile - 1) / kTile * kTile + 2047) / 2048 * 2048;
    if (fit > all) fit = all;
    if (fit < 2048) fit = 2048;
    l.chunk_len = (int)fit;
    l.bytes = codes + std::max((size_t)fit * per_pos4 / 4 + kRefSlack, merge_bytes(G));
    return l;
}

size_t unit_mfma_lds_bytes(int N, int G, bool stash, int S) { return unit_lds(N, G, stash, S).bytes; }

// One launch of one kernel instance.  The dynamic-LDS ceiling is a per-device function
// attribute: it is raised once per device and instance (attr_done, indexed by idx).
struct UnitLaunch {
    std::atomic<bool> *attr_done;
    long long wgs;
    size_t lds;
    hipStream_t s;
    const UnitArgs *a;
    const GroupArgs *ga;
};
constexpr int kUnitInstances = 16;

template <int STASH, bool COOP, bool GROUPED, bool MASKED, bool MAXFREE>
static hipError_t launch_instance(const UnitLaunch &ul, int idx)
{
    auto kern = unit_mfma_kernel<true, STASH, COOP, GROUPED, MASKED, MAXFREE>;
    if (!ul.attr_done[idx].load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kUnitLdsLimit);
        if (e != hipSuccess) return e;
        ul.attr_done[idx].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)ul.wgs), dim3(512), ul.lds, ul.s, *ul.a, *ul.ga);
    return hipGetLastError();
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
    a.arrive = p.arrive;
    a.gcode = (uint8_t *)p.stash_w; a.gref = p.stash_m;
    a.n = n; a.N = p.N; a.G = p.G; a.ntiles = p.ntiles;
    a.S = S; a.split_len = unit_mfma_split_len(p.N, S);
    a.s_active = (n + a.split_len - 1) / a.split_len;
    a.code_stride = (a.split_len + 63) / 64 * 64;
    a.gstride = p.ntiles * kTile;
    const UnitLds l = unit_lds(p.N, p.G, !(p.flags & 1u), S);
    a.merge_off = (int)l.merge_off;
    a.chunk_len = l.chunk_len;
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
    if (lds > kUnitLdsLimit) return hipErrorInvalidValue;
    // With at most a few workgroups per compute unit, ask for more than half of the
    // CU's LDS so that no CU is handed two of them while another one idles.
    const long long wgs = (long long)ga.wgs_per_cache * n_caches;
    if (wgs <= 2 * 256 && lds < 81 * 1024) lds = 81 * 1024;
    if (wgs > 0x7fffffffll) return hipErrorInvalidValue;
    // the dynamic-LDS ceiling is a per-device function attribute: raise it once per device
    // and kernel instance (two host threads that get here together both set it: the call is idempotent, the
    // flags are atomic)
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> attr_done_all[kMaxDevices][kUnitInstances] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    const UnitLaunch ul = {attr_done_all[dev], wgs, lds, s, &a, &ga};
    const bool coop = S > 1, grouped = table != nullptr;
    if (p.max_free) { // one cache, no mask (the API layer admits nothing else)
        if (table || p.masked) return hipErrorInvalidValue;
        if (stash)
            return coop ? launch_instance<kStashLds, true, false, false, true>(ul, 14)
                        : launch_instance<kStashLds, false, false, false, true>(ul, 15);
        return coop ? launch_instance<kStashNone, true, false, false, true>(ul, 12)
                    : launch_instance<kStashNone, false, false, false, true>(ul, 13);
    }
    // the mask only matters where slots are scored (an attention-only cache takes none)
#define LF_PICK(STASH, MASKED, base)                                                                      \
    (coop ? (grouped ? launch_instance<STASH, true, true, MASKED, false>(ul, base + 0)                     \
                     : launch_instance<STASH, true, false, MASKED, false>(ul, base + 1))                   \
          : (grouped ? launch_instance<STASH, false, true, MASKED, false>(ul, base + 2)                    \
                     : launch_instance<STASH, false, false, MASKED, false>(ul, base + 3)))
    if (!stash) return LF_PICK(kStashNone, false, 0);
    if (p.masked) return LF_PICK(kStashLds, true, 4);
    return LF_PICK(kStashLds, false, 8);
#undef LF_PICK
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
