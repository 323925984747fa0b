// A prompt longer than the budget, cut to the budget once before decoding (bf16, head_dim 128).
//
// The paper compresses such a prompt with SnapKV before its own per-step eviction takes over
// (Sec. 4.1, implementation details) and does not restate that procedure.  What is built here, per
// (batch, KV head) unit with its G query heads, T prompt rows, the last W of them the observation
// window and P = T - W the prefix:
//
//   stats    every window query (W x G columns; query j sees rows [0, P + j]) gets its softmax
//            reference and denominator over the rows it sees                       (eq. 1)
//   votes    vote(i) = sum over the W x G columns of alpha(i), for the prefix rows i < P
//   pool     pooled(i) = mean of vote over the `pool` rows centred on i (zero outside the prefix)
//   select   the keep - W prefix rows with the largest pooled vote (lowest row among equals)
//   gather   those rows, in prompt order, then the window, become slots 0 .. keep - 1 of the cache
//
// The two passes over K are multi-query products on the matrix cores with the QUERIES as the A
// operand and the K rows as the B operand: an accumulator register then belongs to (query 4g + v,
// row r of the tile), so a query's running sums stay in one lane (no cross-lane traffic per tile)
// and the per-row vote is a sum over a lane's registers and over the four lane groups.
#include "lf_mfma_stream.h"

namespace lf {

namespace {

constexpr int kCD = 128;       // head_dim
constexpr int kCWaves = 4;     // waves per workgroup
constexpr int kCBlocks = 4;    // 16-column query blocks per wave
constexpr int kColsPerRound = 16 * kCWaves * kCBlocks; // columns one workgroup takes through a span at once

struct CompressArgs {
    const uint16_t *q_window; // [W][units][G][128]
    const uint16_t *Kp, *Vp;  // [units][T][128]
    float *part_m, *part_l;   // [units][nspans][colsP]  per-span softmax state of every column
    float *cq;                // [units][colsP]          reference + log2 denominator of every column
    float *votes;             // [units][Pp]
    float *pooled;            // [units][P]
    int32_t *kept;            // [units][keep]
    uint16_t *Kc, *Vc;        // cache [units][N][128]
    float *lu;                // side array of the matrix-core kernels, or nullptr
    int units, G, T, W, P, Pp, keep, pool, N, lu_stride;
    int cols, colsP, LS, nspans;
    float scale_log2;
};

// Query rows of a wave's NB blocks as A operands: lane (g, r) holds column 16 qb + r, channels 32 c + 8 g .. + 7.
template <int NB> struct QueryBlocks {
    u32x4 q[NB][4];
    __device__ __forceinline__ void load(const CompressArgs &a, int u, int qb0, int g, int r)
    {
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const int col = 16 * (qb0 + b) + r;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                q[b][c] = u32x4{0u, 0u, 0u, 0u};
                if (col < a.cols)
                    q[b][c] = *(const u32x4 *)(a.q_window + (((size_t)(col / a.G) * a.units + u) * a.G + col % a.G) * kCD + 32 * c + 8 * g);
            }
        }
    }
};

struct KRows {
    u32x4 k[4]; // row base + r, channels 32 c + 8 g .. + 7: the B operand of one 16-row tile
};

// K tiles of a span, staged through LDS.  The four waves of a workgroup want the same 16-row tiles as
// operands; if each fetched them for itself, the compute unit's vector-memory path would be the limit of
// both passes (counters: TA_TA_BUSY 85 % / 60 %).  Instead the 256 threads fetch a tile once, 16 bytes per
// thread, park it in a ring of four LDS slots (rows padded to 288 bytes: the stride at which the 16-byte operand
// reads run at the full LDS rate), and every wave reads its operands from there.
// One barrier per tile; the fetch of tile i + 4 is in flight while tile i is used.
struct KRing {
    static constexpr int RS = 288, SLOT = kTile * RS, NSLOT = 4; // 288: the stride at which this read pattern runs at the full LDS rate (timed: two thirds of it at 272, 304, 320)
    unsigned char *ring;   // NSLOT * SLOT bytes of LDS
    const uint16_t *src;   // this thread's 16 bytes of row 0 of the unit's K
    int st_row, st_off, first, last_tile, last_row, g, r;
    __device__ __forceinline__ void init(unsigned char *lds, const uint16_t *Ku, int start, int nt, int last_row_, int tid, int g_, int r_)
    {
        ring = lds; g = g_; r = r_;
        st_row = tid >> 4;
        src = Ku + (tid & 15) * 8;
        st_off = st_row * RS + (tid & 15) * 16;
        first = start; last_tile = nt - 1; last_row = last_row_;
    }
    // rows past the last one: that row again (never used as such)
    __device__ __forceinline__ u32x4 fetch(int ti) const
    {
        return *(const u32x4 *)(src + (size_t)min(first + min(ti, last_tile) * kTile + st_row, last_row) * kCD);
    }
    __device__ __forceinline__ void park(int ti, u32x4 v) const { *(u32x4 *)(ring + (ti % NSLOT) * SLOT + st_off) = v; }
    __device__ __forceinline__ void operands(KRows &t, int ti) const
    {
        const unsigned char *base = ring + (ti % NSLOT) * SLOT + r * RS + 16 * g;
#pragma unroll
        for (int c = 0; c < 4; ++c) t.k[c] = *(const u32x4 *)(base + 64 * c);
    }
    // every thread of the workgroup runs the same nt rounds; use(t, ti) consumes tile ti
    template <typename F> __device__ __forceinline__ void run(int nt, F &&use) const
    {
        if (nt < 1) return;
        u32x4 q0 = fetch(0), q1 = fetch(1);
        park(0, q0);
        park(1, q1);
        q0 = fetch(2);
        q1 = fetch(3);
        __syncthreads();
        KRows ta, tb;
        operands(ta, 0);
        for (int i = 0; i < nt; i += 2) {
            park(i + 2, q0); // fetched two rounds ago
            q0 = fetch(i + 4);
            operands(tb, i + 1);
            use(ta, i);
            __syncthreads();
            if (i + 1 < nt) {
                park(i + 3, q1);
                q1 = fetch(i + 5);
                operands(ta, i + 2);
                use(tb, i + 1);
                __syncthreads();
            }
        }
    }
};

// logits of (query 4g + v of a block, row r of the tile), unscaled
__device__ __forceinline__ f32x4 block_logits(const u32x4 (&q)[4], const KRows &t)
{
    f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < 4; ++c)
        d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, q[c]), __builtin_bit_cast(bf16x8, t.k[c]), d, 0, 0, 0);
    return d;
}

// number of live 16-column blocks among the kCBlocks a wave is responsible for, starting at block qb0
__device__ __forceinline__ int live_blocks(const CompressArgs &a, int qb0)
{
    return min(max((a.cols + 15) / 16 - qb0, 0), kCBlocks);
}

// ---- pass 1: softmax state of NB blocks of columns over one span of rows (NB = 0: a wave without
// columns, which only helps staging the tiles)
template <int NB>
__device__ __forceinline__ void stats_span(const CompressArgs &a, int u, int sp, int qb0, int g, int r, unsigned char *lds)
{
    constexpr int NBA = NB > 0 ? NB : 1;
    QueryBlocks<NBA> Q;
    if (NB > 0) Q.load(a, u, qb0, g, r);
    // column 16 (qb0 + b) + 4 g + v sees rows below lim[b][v]; an unused column sees none
    int lim[NBA][4];
    float m[NBA][4], l[NBA][4];
#pragma unroll
    for (int b = 0; b < NBA; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int col = 16 * (qb0 + b) + 4 * g + v;
            lim[b][v] = col < a.cols ? a.P + col / a.G + 1 : 0;
            m[b][v] = kNoRef;
            l[b][v] = 0.f;
        }

    const int start = sp * a.LS, end = min(start + a.LS, a.T);
    const int nt = (end - start + kTile - 1) / kTile;
    auto consume = [&](const KRows &t, int ti) __attribute__((always_inline)) {
        if (NB == 0) return;
        const int base = start + ti * kTile;
        float x[NBA][4];
#pragma unroll
        for (int b = 0; b < NBA; ++b) {
            const f32x4 d = block_logits(Q.q[b], t);
#pragma unroll
            for (int v = 0; v < 4; ++v) x[b][v] = d[v] * a.scale_log2;
        }
        // Every used column sees every prefix row, so a tile that lies inside the prefix needs no
        // masking (an unused column collects garbage nobody reads); tiles that touch the window or the
        // ragged end take the per-column row limit.
        if (base + kTile > a.P) {
#pragma unroll
            for (int b = 0; b < NBA; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (base + r >= lim[b][v]) x[b][v] = -INFINITY;
        }
        // The reference of a lane's share is raised only when a logit passes it by more than kMaxSlack
        // (weights stay below 2^kMaxSlack); one wave-wide test keeps the common case branch-free.
        bool raise = false;
#pragma unroll
        for (int b = 0; b < NBA; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) raise |= x[b][v] > m[b][v] + kMaxSlack;
        if (__any(raise)) {
#pragma unroll
            for (int b = 0; b < NBA; ++b)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (x[b][v] > m[b][v] + kMaxSlack) {
                        l[b][v] *= fast_exp2(m[b][v] - x[b][v]);
                        m[b][v] = x[b][v];
                    }
        }
#pragma unroll
        for (int b = 0; b < NBA; ++b)
#pragma unroll
            for (int v = 0; v < 4; ++v) l[b][v] += fast_exp2(x[b][v] - m[b][v]);
    };
    KRing ring;
    ring.init(lds, a.Kp + (size_t)u * a.T * kCD, start, nt, a.T - 1, threadIdx.x, g, r);
    ring.run(nt, consume);
    if (NB == 0) return;

    // the 16 lanes of a row group hold the shares of the same four queries
#pragma unroll
    for (int b = 0; b < NBA; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const float M = row16_max(m[b][v]);
            const float L = row16_sum(l[b][v] * fast_exp2(m[b][v] - M));
            const int col = 16 * (qb0 + b) + 4 * g + v;
            if (r == 0 && col < a.cols) {
                const size_t at = ((size_t)u * a.nspans + sp) * a.colsP + col;
                a.part_m[at] = M;
                a.part_l[at] = L;
            }
        }
}

// grid: units x nspans x rounds; workgroup = 4 waves x (up to) 4 blocks x 16 columns
__global__ __launch_bounds__(64 * kCWaves) void compress_stats_kernel(const CompressArgs a)
{
    const int rounds = (a.colsP + kColsPerRound - 1) / kColsPerRound;
    int bid = blockIdx.x;
    const int round = bid % rounds; bid /= rounds;
    const int sp = bid % a.nspans;
    const int u = bid / a.nspans;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, r = lane & 15;
    const int qb0 = (round * kCWaves + wave) * kCBlocks;
    __shared__ __align__(16) unsigned char k_ring[KRing::NSLOT * KRing::SLOT];
    switch (live_blocks(a, qb0)) { // (uniform over a wave; every wave runs the same barriers inside)
    case 4: stats_span<4>(a, u, sp, qb0, g, r, k_ring); break;
    case 3: stats_span<3>(a, u, sp, qb0, g, r, k_ring); break;
    case 2: stats_span<2>(a, u, sp, qb0, g, r, k_ring); break;
    case 1: stats_span<1>(a, u, sp, qb0, g, r, k_ring); break;
    default: stats_span<0>(a, u, sp, qb0, g, r, k_ring); break;
    }
}

// ---- per column: reference + log2 denominator over all spans (+inf for an unused column)
__global__ __launch_bounds__(256) void compress_norm_kernel(const CompressArgs a)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.units * a.colsP) return;
    const int u = (int)(idx / a.colsP), col = (int)(idx % a.colsP);
    float out = INFINITY;
    if (col < a.cols) {
        float M = kNoRef;
        for (int sp = 0; sp < a.nspans; ++sp) M = fmaxf(M, a.part_m[((size_t)u * a.nspans + sp) * a.colsP + col]);
        double Z = 0.0;
        for (int sp = 0; sp < a.nspans; ++sp) {
            const size_t at = ((size_t)u * a.nspans + sp) * a.colsP + col;
            Z += (double)a.part_l[at] * (double)fast_exp2(a.part_m[at] - M);
        }
        out = M + __builtin_amdgcn_logf((float)Z);
    }
    a.cq[idx] = out;
}

// ---- pass 2: votes of the prefix rows of one span, from NB blocks of columns, added into `mine`
// (NB = 0: a wave without columns in this round, which only helps staging the tiles)
template <int NB>
__device__ __forceinline__ void votes_span(const CompressArgs &a, int u, int qb0, int start, int nt, __attribute__((address_space(3))) float *mine, int g, int r, unsigned char *lds)
{
    constexpr int NBA = NB > 0 ? NB : 1;
    QueryBlocks<NBA> Q;
    if (NB > 0) Q.load(a, u, qb0, g, r);
    float cq[NBA][4];
#pragma unroll
    for (int b = 0; b < NBA; ++b)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int col = 16 * (qb0 + b) + 4 * g + v;
            cq[b][v] = col < a.colsP ? a.cq[(size_t)u * a.colsP + col] : INFINITY; // +inf for an unused column: weight 0
        }
    auto consume = [&](const KRows &t, int ti) __attribute__((always_inline)) {
        if (NB == 0) return;
        float w = 0.f;
#pragma unroll
        for (int b = 0; b < NBA; ++b) {
            const f32x4 d = block_logits(Q.q[b], t);
#pragma unroll
            for (int v = 0; v < 4; ++v) w += fast_exp2(fmaf(d[v], a.scale_log2, -cq[b][v])); // alpha, eq. 1
        }
        // every prefix row is seen by every window query.  The four lanes that hold shares of row r add
        // them to the wave's own LDS row with a no-return LDS add: nothing to wait for
        __hip_atomic_fetch_add(&mine[ti * kTile + r], w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    };
    KRing ring;
    ring.init(lds, a.Kp + (size_t)u * a.T * kCD, start, nt, a.P - 1, threadIdx.x, g, r);
    ring.run(nt, consume);
}

// grid: units x nspans2; the workgroup takes every round of columns through its span, each wave
// adding into a row of LDS of its own, and the waves' rows are summed in a fixed order at the end
__global__ __launch_bounds__(64 * kCWaves) void compress_votes_kernel(const CompressArgs a)
{
    extern __shared__ float wave_votes[]; // [kCWaves][LS]
    __shared__ __align__(16) unsigned char k_ring[KRing::NSLOT * KRing::SLOT];
    const int nspans2 = (a.P + a.LS - 1) / a.LS;
    const int sp = blockIdx.x % nspans2, u = blockIdx.x / nspans2;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4, r = lane & 15;
    const int start = sp * a.LS, end = min(start + a.LS, a.P);
    const int nt = (end - start + kTile - 1) / kTile;
    __attribute__((address_space(3))) float *mine = (__attribute__((address_space(3))) float *)wave_votes + (size_t)wave * a.LS;
    for (int i = lane; i < a.LS; i += 64) mine[i] = 0.f;

    const int rounds = (a.colsP + kColsPerRound - 1) / kColsPerRound;
    for (int round = 0; round < rounds; ++round) {
        const int qb0 = (round * kCWaves + wave) * kCBlocks;
        switch (live_blocks(a, qb0)) { // (uniform over a wave; every wave runs the same barriers inside)
        case 4: votes_span<4>(a, u, qb0, start, nt, mine, g, r, k_ring); break;
        case 3: votes_span<3>(a, u, qb0, start, nt, mine, g, r, k_ring); break;
        case 2: votes_span<2>(a, u, qb0, start, nt, mine, g, r, k_ring); break;
        case 1: votes_span<1>(a, u, qb0, start, nt, mine, g, r, k_ring); break;
        default: votes_span<0>(a, u, qb0, start, nt, mine, g, r, k_ring); break;
        }
        __syncthreads(); // the ring is reused by the next round of columns
    }
    __syncthreads();
    for (int i = threadIdx.x; i < end - start; i += 64 * kCWaves) {
        float s = wave_votes[i];
#pragma unroll
        for (int w = 1; w < kCWaves; ++w) s += wave_votes[(size_t)w * a.LS + i];
        a.votes[(size_t)u * a.Pp + start + i] = s;
    }
}

// ---- pooling: mean over the `pool` rows centred on i, rows outside the prefix counting as zero
__global__ __launch_bounds__(256) void compress_pool_kernel(const CompressArgs a)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (long long)a.units * a.P) return;
    const int u = (int)(idx / a.P), i = (int)(idx % a.P);
    const float *v = a.votes + (size_t)u * a.Pp;
    const int h = a.pool / 2;
    float s = 0.f;
    for (int j = max(i - h, 0); j <= min(i + h, a.P - 1); ++j) s += v[j];
    a.pooled[idx] = s / (float)a.pool;
}

// ---- selection: one workgroup per unit.  Pooled votes are non-negative, so their bit patterns
// order like the values: a radix search (8 bits a round, from the top) finds the bit pattern of
// the kp-th largest; rows above it are kept, rows equal to it lowest row first until kp are
// taken, and the kept rows are written out in ascending row order, followed by the window.
constexpr int kSelThreads = 1024;
__global__ __launch_bounds__(kSelThreads) void compress_select_kernel(const CompressArgs a)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_prefix, s_need;
    __shared__ uint32_t wave_eq[kSelThreads / 64], wave_keep[kSelThreads / 64];
    __shared__ uint32_t base_eq, base_keep;
    const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int P = a.P, kp = a.keep - a.W;
    const uint32_t *bits = (const uint32_t *)(a.pooled + (size_t)u * P);
    int32_t *kept = a.kept + (size_t)u * a.keep;

    if (kp > 0 && kp < P) {
        if (tid == 0) { s_prefix = 0u; s_need = (uint32_t)kp; }
        for (int shift = 24; shift >= 0; shift -= 8) {
            if (tid < 256) hist[tid] = 0u;
            __syncthreads();
            const uint32_t prefix = s_prefix;
            const uint32_t himask = shift == 24 ? 0u : 0xffffffffu << (shift + 8);
            for (int i = tid; i < P; i += kSelThreads) {
                const uint32_t x = bits[i] & 0x7fffffffu;
                if ((x & himask) == prefix) atomicAdd(&hist[(x >> shift) & 255u], 1u);
            }
            __syncthreads();
            if (tid == 0) { // from the top bin down: the bin in which the kp-th largest falls
                uint32_t need = s_need;
                int bin = 255;
                for (; bin > 0; --bin) {
                    if (hist[bin] >= need) break;
                    need -= hist[bin];
                }
                s_need = need;
                s_prefix = prefix | ((uint32_t)bin << shift);
            }
            __syncthreads();
        }
    }
    // thr: bit pattern of the kp-th largest; need_eq rows equal to it are kept, lowest first
    uint32_t thr, need_eq;
    if (kp <= 0) { thr = 0xffffffffu; need_eq = 0u; }        // nothing from the prefix
    else if (kp >= P) { thr = 0u; need_eq = (uint32_t)P; }    // all of it
    else { thr = s_prefix; need_eq = s_need; }
    if (tid == 0) { base_eq = 0u; base_keep = 0u; }
    __syncthreads();

    for (int c0 = 0; c0 < P; c0 += kSelThreads) {
        const int i = c0 + tid;
        const uint32_t x = i < P ? bits[i] & 0x7fffffffu : 0u;
        const bool gt = i < P && x > thr && kp > 0;
        const bool eq = i < P && x == thr && kp > 0;
        const uint64_t b_eq = __ballot(eq);
        const uint32_t below = (uint32_t)__popcll(b_eq & ((1ull << lane) - 1ull));
        if (lane == 0) wave_eq[wave] = (uint32_t)__popcll(b_eq);
        __syncthreads();
        uint32_t eq_rank = base_eq + below;
        for (int w = 0; w < wave; ++w) eq_rank += wave_eq[w];
        const bool keep_row = gt || (eq && eq_rank < need_eq);
        const uint64_t b_k = __ballot(keep_row);
        const uint32_t kbelow = (uint32_t)__popcll(b_k & ((1ull << lane) - 1ull));
        if (lane == 0) wave_keep[wave] = (uint32_t)__popcll(b_k);
        __syncthreads();
        uint32_t pos = base_keep + kbelow;
        for (int w = 0; w < wave; ++w) pos += wave_keep[w];
        if (keep_row && pos < (uint32_t)kp) kept[pos] = i;
        __syncthreads();
        if (tid == 0) {
            uint32_t te = 0u, tk = 0u;
            for (int w = 0; w < kSelThreads / 64; ++w) { te += wave_eq[w]; tk += wave_keep[w]; }
            base_eq += te;
            base_keep += tk;
        }
        __syncthreads();
    }
    for (int j = tid; j < a.W; j += kSelThreads) kept[max(kp, 0) + j] = P + j; // the window is always kept
}

// ---- gather: one 16-lane row per (unit, destination slot)
__global__ __launch_bounds__(256) void compress_gather_kernel(const CompressArgs a)
{
    const int lane16 = threadIdx.x & 15;
    const long long total = (long long)a.units * a.keep;
    for (long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4); row < total; row += (long long)gridDim.x * 16) {
        const int u = (int)(row / a.keep), slot = (int)(row % a.keep);
        int src = a.kept[row];
        src = min(max(src, 0), a.T - 1); // the selection writes rows of the prompt only; keeps a stray value harmless
        const u32x4 kk = *(const u32x4 *)(a.Kp + ((size_t)u * a.T + src) * kCD + 8 * lane16);
        const u32x4 vv = *(const u32x4 *)(a.Vp + ((size_t)u * a.T + src) * kCD + 8 * lane16);
        *(u32x4 *)(a.Kc + ((size_t)u * a.N + slot) * kCD + 8 * lane16) = kk;
        *(u32x4 *)(a.Vc + ((size_t)u * a.N + slot) * kCD + 8 * lane16) = vv;
        float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                   fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
        a1 = row16_sum(a1);
        if (lane16 == 0 && a.lu) a.lu[(size_t)u * a.lu_stride + (slot & ~15) + pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
    }
}

} // namespace

void compress_geometry(int units, int T, int *LS, int *nspans)
{
    // spans of at most 2048 rows, shorter (down to 256) while the grid would not fill the chip
    int ls = 2048;
    while (ls > 256 && (long long)units * ((T + ls - 1) / ls) < 1024) ls /= 2;
    *LS = ls;
    *nspans = (T + ls - 1) / ls;
}

static size_t up256(size_t x) { return (x + 255) / 256 * 256; }

CompressLayout compress_layout(int units, int G, int T, int W, int keep_max)
{
    CompressLayout l;
    int LS, nspans;
    compress_geometry(units, T, &LS, &nspans);
    const int cols = W * G, colsP = (cols + 15) / 16 * 16;
    const int P = T - W, Pp = (P + kTile - 1) / kTile * kTile;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = up256(off + bytes); return o; };
    l.off_part_m = take(sizeof(float) * (size_t)units * nspans * colsP);
    l.off_part_l = take(sizeof(float) * (size_t)units * nspans * colsP);
    l.off_cq = take(sizeof(float) * (size_t)units * colsP);
    l.off_votes = take(sizeof(float) * (size_t)units * (Pp > 0 ? Pp : 1));
    l.off_pooled = take(sizeof(float) * (size_t)units * (P > 0 ? P : 1));
    l.off_kept = take(sizeof(int32_t) * (size_t)units * keep_max);
    l.total = off;
    return l;
}

hipError_t launch_compress_prompt(const Plan &p, int T, int W, int keep, int pool, const void *q_window,
                                  const void *k_prompt, const void *v_prompt, void *scratch, hipStream_t s)
{
    const CompressLayout l = compress_layout(p.units, p.G, T, W, p.N);
    char *sc = (char *)scratch;
    CompressArgs a;
    a.q_window = (const uint16_t *)q_window;
    a.Kp = (const uint16_t *)k_prompt; a.Vp = (const uint16_t *)v_prompt;
    a.part_m = (float *)(sc + l.off_part_m); a.part_l = (float *)(sc + l.off_part_l);
    a.cq = (float *)(sc + l.off_cq);
    a.votes = (float *)(sc + l.off_votes);
    a.pooled = (float *)(sc + l.off_pooled);
    a.kept = (int32_t *)(sc + l.off_kept);
    a.Kc = (uint16_t *)p.k_cache; a.Vc = (uint16_t *)p.v_cache;
    a.lu = p.lu;
    a.units = p.units; a.G = p.G; a.T = T; a.W = W; a.P = T - W; a.Pp = (a.P + kTile - 1) / kTile * kTile;
    a.keep = keep; a.pool = pool; a.N = p.N; a.lu_stride = p.ntiles * kTile;
    a.cols = W * p.G; a.colsP = (a.cols + 15) / 16 * 16;
    compress_geometry(p.units, T, &a.LS, &a.nspans);
    a.scale_log2 = 1.4426950408889634f / sqrtf(128.f);

    hipError_t e = hipSuccess;
    const int rounds = (a.colsP + kColsPerRound - 1) / kColsPerRound;
    if (a.P > 0) {
        hipLaunchKernelGGL(compress_stats_kernel, dim3((unsigned)((long long)p.units * a.nspans * rounds)), dim3(64 * kCWaves), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(compress_norm_kernel, dim3((unsigned)(((long long)p.units * a.colsP + 255) / 256)), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        const int nspans2 = (a.P + a.LS - 1) / a.LS;
        hipLaunchKernelGGL(compress_votes_kernel, dim3((unsigned)((long long)p.units * nspans2)), dim3(64 * kCWaves),
                           sizeof(float) * kCWaves * a.LS, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(compress_pool_kernel, dim3((unsigned)(((long long)p.units * a.P + 255) / 256)), dim3(256), 0, s, a);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(compress_select_kernel, dim3(p.units), dim3(kSelThreads), 0, s, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    long long blocks = ((long long)p.units * keep + 15) / 16;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(compress_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace lf
