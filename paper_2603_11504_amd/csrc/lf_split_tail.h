// Head and tail of the split-K kernels: slot insert by the workgroup that owns the slot,
// and the cross-split finish run by whichever workgroup of a unit finishes last.
//
// With these two pieces every split-K path is a single launch per decode step:
//   head   the workgroup whose slot range holds the pending slot writes k_new / v_new
//          there before anyone in the workgroup streams the row        (Fig. 2 left)
//   tail   each workgroup publishes its partial softmax state and screening stash, then
//          bumps a per-unit counter; the last one to arrive merges the partials into the
//          output (eq. 1), screens the stash, re-scores the candidates exactly in double
//          precision and writes the next pending slot (Sec. 3.2; Alg. 1 post-processing).
// No workgroup ever waits for another: the pattern cannot deadlock whatever the
// dispatch order.
#pragma once
#include "lf_device.h"
#include "lf_host.h"

namespace lf {

__host__ __device__ constexpr __forceinline__ int tail_pos_of_slot(int s) { return 4 * ((s >> 1) & 3) + 2 * ((s >> 3) & 1) + (s & 1); }
__host__ __device__ constexpr __forceinline__ int tail_slot_of_pos(int p) { return 8 * ((p >> 1) & 1) + 2 * (p >> 2) + (p & 1); }

template <typename T> struct SplitTailArgs {
    T *Kc, *Vc;               // caches [units][N][D]
    const T *q, *k_new, *v_new;
    T *out, *q_last;
    int32_t *pending, *evict_idx, *arrive; // arrive: per-unit arrival counter, zero between steps
    float *part_m, *part_l, *part_o;       // [units][C][G], [units][C][G], [units][C][G][D]
    uint16_t *stash_w;                     // [units][ntiles][G][16] bf16
    float *stash_m;                        // [units][ntiles][G]
    float *fin_m, *fin_l;                  // [units][G]
    float *lu;                             // [units][ntiles*16] log2 ||v||_1 (position order); null if attention-only
    int n, N, G, C, c_active, ntiles, L;
    int attention_only, pos_order;
    int fused_tail; // 1: the last workgroup of a unit to arrive finishes it; 0: a finish launch follows
    int masked;     // explicit mask in force: NaN entries of lu mark invalid slots
};

// The fused tail needs a device-wide release/acquire per workgroup, which on this chip
// writes back each XCD's L2: cheap for a few dozen workgroups, ruinous for thousands
// (measured: 82 -> 517 us at 2048 workgroups).  Large grids take a separate finish launch.
inline bool split_uses_fused_tail(const Plan &p, int n, int n_caches = 1)
{
    const long long wgs = (long long)p.units * ((n + p.L - 1) / p.L) * n_caches;
    return wgs <= 256;
}

// Several caches of one geometry and fill level in one grid: per-cache pointers come from a
// device table of SplitTailArgs, the step's tensors from base pointers plus a stride per
// cache (in elements).  table == nullptr: a single cache, arguments as passed.
struct SplitGroup {
    const void *table;
    int per_cache;     // workgroups per cache in this launch
    long long q_stride, kv_stride, ev_stride;
};

template <typename T>
inline SplitTailArgs<T> make_tail_args(const Plan &p, const StepIo &io, int n, int n_caches = 1)
{
    SplitTailArgs<T> a;
    a.Kc = (T *)p.k_cache; a.Vc = (T *)p.v_cache;
    a.q = (const T *)io.q; a.k_new = (const T *)io.k_new; a.v_new = (const T *)io.v_new;
    a.out = (T *)io.out; a.q_last = (T *)p.q_last;
    a.pending = p.pending; a.evict_idx = io.evict_idx; a.arrive = p.arrive;
    a.part_m = p.part_m; a.part_l = p.part_l; a.part_o = p.part_o;
    a.stash_w = p.stash_w; a.stash_m = p.stash_m;
    a.fin_m = p.fin_m; a.fin_l = p.fin_l;
    // the vector-ALU kernels need the side array only while an explicit mask is in force
    a.lu = ((p.use_mfma || p.masked) && !(p.flags & 1u)) ? p.lu : nullptr;
    a.masked = p.masked ? 1 : 0;
    a.n = n; a.N = p.N; a.G = p.G; a.C = p.C; a.c_active = (n + p.L - 1) / p.L; a.ntiles = p.ntiles; a.L = p.L;
    a.attention_only = (p.flags & 1u) ? 1 : 0;
    a.pos_order = p.use_mfma ? 1 : 0;
    a.fused_tail = split_uses_fused_tail(p, n, n_caches) ? 1 : 0;
    return a;
}

inline SplitGroup make_split_group(const Plan &p, const void *table, int per_cache)
{
    SplitGroup g;
    g.table = table;
    g.per_cache = per_cache;
    g.q_stride = (long long)p.units * p.G * p.D;
    g.kv_stride = (long long)p.units * p.D;
    g.ev_stride = p.units;
    return g;
}

// Workgroup's index within its cache; for a group, `a` is switched to that cache first.
template <typename T>
__device__ __forceinline__ int split_group_select(SplitTailArgs<T> &a, const SplitGroup &gr)
{
    int blk = blockIdx.x;
    if (gr.table) {
        const int ci = blk / gr.per_cache;
        blk -= ci * gr.per_cache;
        const SplitTailArgs<T> *t = (const SplitTailArgs<T> *)gr.table + ci;
        a.Kc = t->Kc; a.Vc = t->Vc; a.q_last = t->q_last;
        a.pending = t->pending; a.arrive = t->arrive;
        a.part_m = t->part_m; a.part_l = t->part_l; a.part_o = t->part_o;
        a.stash_w = t->stash_w; a.stash_m = t->stash_m;
        a.fin_m = t->fin_m; a.fin_l = t->fin_l;
        a.lu = a.lu ? t->lu : nullptr; // whether it is used is this step's decision, not the table's
        a.q += ci * gr.q_stride;
        a.out += ci * gr.q_stride;
        if (a.k_new) a.k_new += ci * gr.kv_stride;
        if (a.v_new) a.v_new += ci * gr.kv_stride;
        if (a.evict_idx) a.evict_idx += ci * gr.ev_stride;
    }
    return blk;
}

// ---- head: executed by all 256 threads of the workgroup (unit u, split c)
template <typename T, int D>
__device__ __forceinline__ void split_head_insert(const SplitTailArgs<T> &a, int u, int c)
{
    if (a.attention_only) return;
    const int slot = a.pending[u];
    if (slot < 0 || slot >= a.N || slot / a.L != c) return; // uniform over the workgroup
    __shared__ float part[4];
    const int tid = threadIdx.x;
    float a1 = 0.f;
    if (tid < D) {
        a.Kc[((size_t)u * a.N + slot) * D + tid] = a.k_new[(size_t)u * D + tid];
        const T v = a.v_new[(size_t)u * D + tid];
        a.Vc[((size_t)u * a.N + slot) * D + tid] = v;
        a1 = fabsf(to_f32(v));
    }
    if (a.lu) { // side array: log2 ||v||_1 for the matrix-core kernels; any non-NaN value says "valid"
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) a1 += __shfl_xor(a1, off);
        if ((tid & 63) == 0) part[tid >> 6] = a1;
        __syncthreads();
        if (tid == 0)
            a.lu[(size_t)u * a.ntiles * kTile + (slot & ~15) + tail_pos_of_slot(slot & 15)] =
                __builtin_amdgcn_logf(part[0] + part[1] + part[2] + part[3]);
    }
    __threadfence_block();
    __syncthreads(); // the row is in place before any wave of this workgroup loads it
}

__device__ __forceinline__ double tail_wave_sum(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// exact LongFlowScore of one slot in double precision, by a whole wave (eq. 6, heads summed)
template <typename T, int D>
__device__ double tail_exact_score(const T *__restrict__ krow, const T *__restrict__ vrow,
                                   const T *__restrict__ qu, int G, const float *sM, const float *sL,
                                   int lane)
{
    constexpr int PER = D / 64;
    double kd[PER], l1 = 0.0;
#pragma unroll
    for (int e = 0; e < PER; ++e) {
        kd[e] = (double)to_f32(krow[lane * PER + e]);
        l1 += fabs((double)to_f32(vrow[lane * PER + e]));
    }
    l1 = tail_wave_sum(l1);
    const double scale_log2 = 1.4426950408889634074 / sqrt((double)D);
    double acc = 0.0;
    for (int h = 0; h < G; ++h) {
        double dot = 0.0;
#pragma unroll
        for (int e = 0; e < PER; ++e) dot += (double)to_f32(qu[(size_t)h * D + lane * PER + e]) * kd[e];
        dot = tail_wave_sum(dot);
        acc += exp2(dot * scale_log2 - (double)sM[h]) / (double)sL[h];
    }
    return acc * l1;
}

// approximate scores of the 8 slots of a half tile from the bf16 stash
__device__ __forceinline__ void tail_screen8(const uint16_t *sw, const float *smt, int tile, int half, int G,
                                             const float *sM, const float *sL, float *sc)
{
#pragma unroll
    for (int e = 0; e < 8; ++e) sc[e] = 0.f;
    for (int h = 0; h < G; ++h) {
        const u32x4 w = *(const u32x4 *)(sw + ((size_t)tile * G + h) * kTile + half * 8);
        const float f = fast_exp2(smt[(size_t)tile * G + h] - sM[h]) / sL[h];
        sc[0] = fmaf(bf16_lo(w.x), f, sc[0]); sc[1] = fmaf(bf16_hi(w.x), f, sc[1]);
        sc[2] = fmaf(bf16_lo(w.y), f, sc[2]); sc[3] = fmaf(bf16_hi(w.y), f, sc[3]);
        sc[4] = fmaf(bf16_lo(w.z), f, sc[4]); sc[5] = fmaf(bf16_hi(w.z), f, sc[5]);
        sc[6] = fmaf(bf16_lo(w.w), f, sc[6]); sc[7] = fmaf(bf16_hi(w.w), f, sc[7]);
    }
}

// ---- finish of unit u by one 256-thread workgroup
template <typename T, int D>
__device__ void split_finish_unit(const SplitTailArgs<T> &a, int u)
{
    __shared__ float sM[kMaxGroup], sL[kMaxGroup];
    __shared__ float sW[kMaxSplits][kMaxGroup];
    __shared__ float red_v[4];
    __shared__ double best_v[4];
    __shared__ int best_i[4];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = a.G, n = a.n, N = a.N;
    const size_t pb = (size_t)u * a.C * G;
    const T *qu = a.q + (size_t)u * G * D;

    if (tid < G) {
        float M = -INFINITY;
        for (int c = 0; c < a.c_active; ++c) M = fmaxf(M, a.part_m[pb + (size_t)c * G + tid]);
        float Ls = 0.f;
        for (int c = 0; c < a.c_active; ++c) {
            const float w = merge_weight(a.part_m[pb + (size_t)c * G + tid], M);
            sW[c][tid] = w;
            Ls += w * a.part_l[pb + (size_t)c * G + tid];
        }
        sM[tid] = M;
        sL[tid] = Ls;
        a.fin_m[(size_t)u * G + tid] = M;
        a.fin_l[(size_t)u * G + tid] = Ls;
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += 256) {
        const int h = idx / D, d = idx % D;
        float acc = 0.f;
        for (int c = 0; c < a.c_active; ++c) acc += sW[c][h] * a.part_o[(pb + (size_t)c * G + h) * D + d];
        store_elem(a.out + ((size_t)u * G + h) * D + d, acc / sL[h]);
        a.q_last[(size_t)u * G * D + idx] = qu[idx]; // kept for longflow_scores()
    }
    if (a.attention_only) return;
    if (n < N) {
        if (tid == 0) {
            a.pending[u] = n;
            if (a.evict_idx) a.evict_idx[u] = n;
        }
        return;
    }

    // ---- explicit mask: an invalid slot (NaN in the side array) takes the next token before
    // anything is evicted; the slot this step filled may still read stale and is skipped
    if (a.masked) {
        __shared__ int hole_w[4];
        const float *lu_u = a.lu + (size_t)u * a.ntiles * kTile;
        const int ins_slot = a.pending[u];
        int best = 0x7fffffff;
        for (int p = tid; p < a.ntiles * kTile; p += 256) {
            const float x = lu_u[p];
            const int slot = (p & ~15) + tail_slot_of_pos(p & 15);
            if (x != x && slot < N && slot != ins_slot) best = min(best, slot);
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) best = min(best, __shfl_xor(best, off));
        if (lane == 0) hole_w[wave] = best;
        __syncthreads();
        best = min(min(hole_w[0], hole_w[1]), min(hole_w[2], hole_w[3]));
        if (best != 0x7fffffff) {
            if (tid == 0) {
                a.pending[u] = best;
                if (a.evict_idx) a.evict_idx[u] = best;
            }
            return;
        }
    }

    // ---- screening pass 1: approximate scores from the stash, block minimum
    const int nhalf = 2 * ((n + kTile - 1) / kTile);
    const int iters = (nhalf + 255) / 256;
    const uint16_t *sw = a.stash_w + (size_t)u * a.ntiles * G * kTile;
    const float *smt = a.stash_m + (size_t)u * a.ntiles * G;
    float vmin = INFINITY;
    for (int it = 0; it < iters; ++it) {
        const int item = it * 256 + tid;
        if (item < nhalf) {
            const int tile = item >> 1, half = item & 1;
            float sc[8];
            tail_screen8(sw, smt, tile, half, G, sM, sL, sc);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int in_tile = half * 8 + e;
                const int slot = tile * kTile + (a.pos_order ? tail_slot_of_pos(in_tile) : in_tile);
                if (slot < n) vmin = fminf(vmin, sc[e]);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) vmin = fminf(vmin, __shfl_xor(vmin, off));
    if (lane == 0) red_v[wave] = vmin;
    __syncthreads();
    const float smin = fminf(fminf(red_v[0], red_v[1]), fminf(red_v[2], red_v[3]));
    // stash values carry relative error <= 2^-9 (bf16 rounding) plus fp32 noise, and an
    // absolute error <= 2^-121 where they underflow: everything that could be the true
    // minimum lies below this threshold
    const float thr = smin * (1.0f + 0.0078125f) + 7.5e-37f;

    // ---- pass 2: exact scores of the candidates, wave-cooperative
    double bv = INFINITY;
    int bi = 0x7fffffff;
    const T *Ku = a.Kc + (size_t)u * N * D;
    const T *Vu = a.Vc + (size_t)u * N * D;
    for (int it = 0; it < iters; ++it) {
        const int item = it * 256 + tid;
        const int tile = item >> 1, half = item & 1;
        float sc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) sc[e] = INFINITY;
        if (item < nhalf) tail_screen8(sw, smt, tile, half, G, sM, sL, sc);
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int in_tile = half * 8 + e;
            const int slot = tile * kTile + (a.pos_order ? tail_slot_of_pos(in_tile) : in_tile);
            const bool cand = (item < nhalf) && (slot < n) && (sc[e] <= thr);
            unsigned long long bal = __ballot(cand);
            while (bal) {
                const int src = __ffsll((long long)bal) - 1;
                bal &= bal - 1;
                const int cs = __shfl(slot, src);
                // scores are >= 0 and ties go to the lower slot: behind an exact zero nothing can win
                // (keeps a unit of zero-norm value rows, e.g. a padded sequence, from re-scoring every slot)
                if (bv == 0.0 && cs > bi) continue;
                const double v = tail_exact_score<T, D>(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qu, G, sM, sL, lane);
                if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
            }
        }
    }
    if (lane == 0) { best_v[wave] = bv; best_i[wave] = bi; }
    __syncthreads();
    if (tid == 0) {
        double v = best_v[0];
        int i = best_i[0];
        for (int w = 1; w < 4; ++w)
            if (best_v[w] < v || (best_v[w] == v && best_i[w] < i)) { v = best_v[w]; i = best_i[w]; }
        if (i < 0 || i >= N) i = 0; // non-finite scores: keep the slot in range
        a.pending[u] = i;
        if (a.evict_idx) a.evict_idx[u] = i;
    }
}

// ---- tail: call after the workgroup's partials and stash have been written
template <typename T, int D>
__device__ __forceinline__ void split_tail(const SplitTailArgs<T> &a, int u)
{
    if (a.c_active == 1) {
        // the unit's only workgroup: nobody to wait for, and what it just wrote it reads back
        // itself -- workgroup-level ordering is enough, no device-wide fence, no counter
        __threadfence_block();
        __syncthreads();
        split_finish_unit<T, D>(a, u);
        return;
    }
    if (!a.fused_tail) return;
    __shared__ int s_last;
    __threadfence(); // this thread's partials/stash are visible device-wide ...
    __syncthreads();
    if (threadIdx.x == 0) s_last = (atomicAdd(&a.arrive[u], 1) == a.c_active - 1); // ... before the arrival counts
    __syncthreads();
    if (!s_last) return;
    __threadfence(); // see what the other workgroups published
    split_finish_unit<T, D>(a, u);
    if (threadIdx.x == 0) a.arrive[u] = 0; // ready for the next step (stream order covers visibility)
}

// stand-alone finish for large grids: one workgroup per unit
template <typename T, int D>
__global__ __launch_bounds__(256) void split_finish_kernel(const SplitTailArgs<T> a_in, const SplitGroup gr)
{
    SplitTailArgs<T> a = a_in;
    const int u = split_group_select(a, gr);
    split_finish_unit<T, D>(a, u);
}

// gr.per_cache of the main launch is units * c_active; the finish grid has one workgroup per unit
template <typename T, int D>
inline hipError_t launch_split_finish(const SplitTailArgs<T> &a, int units, SplitGroup gr, int n_caches, hipStream_t s)
{
    gr.per_cache = units;
    hipLaunchKernelGGL((split_finish_kernel<T, D>), dim3(units * n_caches), dim3(256), 0, s, a, gr);
    return hipGetLastError();
}

} // namespace lf
