// Fill phase in bulk (bf16, head_dim 128): the next T tokens of a cache that still has room.
//
// While a cache is filling nothing is evicted, so consecutive decode steps depend on each
// other only through the rows they append: token t attends to the rows present after its
// own insert (Sec. 2.1).  All rows are therefore written first, and the queries then go
// through attention several at a time, each column of the S^T = K Q^T product carrying one
// (token, head) pair with its own causal row limit.  A 16-column product holds floor(16 / G)
// tokens, a wave takes NB = 3 such products through every pair of tiles, and the eight waves of
// a workgroup take eight different sets of tokens through the same tiles, staged once in LDS: HBM
// delivers the cache once per 24 * floor(16 / G) tokens
// instead of once per token, and the kernel is bound by arithmetic, not by memory.  Being so, it
// takes K in the natural operand layout (half the matrix instructions for the logits).
#include "lf_mfma_stream.h"

namespace lf {

struct FillArgs {
    uint16_t *Kc, *Vc;
    float *lu;         // side array of the matrix-core kernels: log2 ||v||_1, tile position order
    const uint16_t *q, *k_new, *v_new; // [T][units][G][128], [T][units][128]
    uint16_t *out;     // [T][units][G][128]
    int n0;            // valid rows before the call
    int Tb;            // tokens inserted and attended here
    int N, G, units, lu_stride;
    int qpb;           // tokens per 16-column product = 16 / G
    float scale_log2;
};

// One 16-lane row per (token, unit): K and V rows into slot n0 + t, log2 ||v||_1 beside them.
__global__ __launch_bounds__(256) void fill_insert_kernel(const FillArgs a)
{
    const int lane16 = threadIdx.x & 15;
    const long long total = (long long)a.Tb * a.units;
    for (long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4); row < total; row += (long long)gridDim.x * 16) {
        const int u = (int)(row % a.units), slot = a.n0 + (int)(row / a.units);
        const u32x4 kk = *(const u32x4 *)(a.k_new + (size_t)row * 128 + 8 * lane16);
        const u32x4 vv = *(const u32x4 *)(a.v_new + (size_t)row * 128 + 8 * lane16);
        *(u32x4 *)(a.Kc + ((size_t)u * a.N + slot) * 128 + 8 * lane16) = kk;
        *(u32x4 *)(a.Vc + ((size_t)u * a.N + slot) * 128 + 8 * lane16) = vv;
        float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                   fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
        a1 = row16_sum(a1);
        if (lane16 == 0 && a.lu) a.lu[(size_t)u * a.lu_stride + (slot & ~15) + pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
    }
}

// One workgroup = one (unit, group of NWV * NB * qpb consecutive tokens).  Each of its NWV waves owns
// NB * qpb of those tokens outright (no wave ever merges with another) and takes them through every tile
// of the rows they see.  The tiles are staged through LDS: the 512 threads of the workgroup fetch each
// K/V tile from device memory once (16 bytes per thread and tile), park it in a ring of four LDS slots,
// and every wave takes its MFMA operands from there.  (When every wave fetched every tile for itself the
// caches served seven of the eight fetches, but each still went through the compute unit's vector-memory
// path, and the counters showed that path -- TA_TA_BUSY 94 % -- not HBM or the matrix pipe as the limit:
// 6.7 M tokens/s against 9.9 M this way on a 64 x 4 x 8192-slot cache.)  Rows are padded in LDS (288 bytes for K, 320 for V: see the constants)
// so that the 16-byte operand reads run at the full LDS rate.  One barrier per pair of tiles; the fetches of tiles i + 4
// and i + 5 are issued while tiles i and i + 1 are computed, two registers of a thread carry them.  (Three products a wave
// need 256 registers and four spilled dwords; measured 14 % faster than two products without a spill.)
template <int NB, int NWV>
__global__ __launch_bounds__(64 * NWV) void fill_attend_kernel(const FillArgs a)
{
    static_assert(NWV == 8, "one 16-byte fetch per thread and tile: 512 threads for 8 KiB of K and V");
    // row strides in LDS, found by timing the two operand read patterns on this chip (ds_read_b128, eight waves): the K
    // pattern (16 rows x 16 bytes per quarter-wave) runs at full LDS rate at 288 bytes and at two thirds of it at 272,
    // 304, 320 ...; the V pattern (256 contiguous bytes per quarter-wave, quarter-waves four rows apart) at 320 only
    constexpr int D = 128, RSK = 288, RSV = 320, VOFF = kTile * RSK, SLOT = kTile * (RSK + RSV), NSLOT = 4;
    typedef MfmaStreamer<1, false, kStashNone, false, true, false, true> Streamer;
    __shared__ __align__(16) unsigned char ring[NSLOT * SLOT];
    const int G = a.G, units = a.units, QW = NB * a.qpb;
    const int ngroups = (a.Tb + NWV * QW - 1) / (NWV * QW);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, r = lane & 15;
    // late tokens see the most rows: their groups go first
    const int qg = ngroups - 1 - (int)(blockIdx.x / units), u = blockIdx.x % units;
    const int t0 = (qg * NWV + wave) * QW;
    const bool has_tokens = t0 < a.Tb; // the last group may be short of waves: those only help staging
    const int tl = min(t0 + QW, a.Tb) - 1;
    const int n_max = has_tokens ? a.n0 + tl + 1 : 0;                  // rows this wave's tokens see
    const int wg_nmax = a.n0 + min((qg + 1) * NWV * QW, a.Tb);         // rows the workgroup's last token sees
    const int nt = (wg_nmax + kTile - 1) / kTile;
    const int qi = r / G, h_of_r = r % G;

    Streamer st[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int t = t0 + nb * a.qpb + qi;
        const bool used = has_tokens && qi < a.qpb && t <= tl;
        st[nb].init_column(used ? (g_cu16p)(a.q + (((size_t)t * units + u) * G + h_of_r) * D) : (g_cu16p) nullptr, a.n0 + t + 1, lane, a.scale_log2);
        st[nb].start = 0;
        st[nb].end = n_max;
    }

    // staging role of this thread: 16 bytes of row st_row of the K tile (threads 0..255) or the V tile
    const int st_row = (tid & 255) >> 4, st_chunk = tid & 15;
    const g_cu16p src = (g_cu16p)((tid < 256 ? a.Kc : a.Vc) + (size_t)u * a.N * D) + st_chunk * 8;
    const int st_off = (tid < 256 ? st_row * RSK : VOFF + st_row * RSV) + st_chunk * 16;
    auto fetch = [&](int ti) __attribute__((always_inline)) { // rows past the last one the workgroup sees: that row again
        return *(g_cu32x4p)(src + (size_t)min(min(ti, nt - 1) * kTile + st_row, wg_nmax - 1) * D);
    };
    auto park = [&](int ti, u32x4 v) __attribute__((always_inline)) { *(u32x4 *)(ring + (ti % NSLOT) * SLOT + st_off) = v; };
    // operands of tile ti from LDS, in the layouts the streaming core computes from (natural K layout)
    auto operands = [&](TileRegs &t, int ti) __attribute__((always_inline)) {
        const unsigned char *base = ring + (ti % NSLOT) * SLOT;
#pragma unroll
        for (int c = 0; c < 4; ++c) t.k[c >> 1][c & 1] = *(const u32x4 *)(base + r * RSK + 64 * c + 16 * g);
#pragma unroll
        for (int e = 0; e < 4; ++e) t.v[e] = *(const u32x4 *)(base + VOFF + (4 * g + e) * RSV + 16 * r);
    };
    const int first_limit = a.n0 + t0 + 1; // rows the wave's first token sees; later tokens see more
    // Two tiles at a time: the logits of both tiles and both products go to the matrix pipe first, then the
    // weights of the first tile, of the second (which may still move the reference: it rescales the first's),
    // and one P V product over the 32 slots of the pair.
    auto compute_pair = [&](TileRegs &t0r, TileRegs &t1r, int ti) __attribute__((always_inline)) {
        if (ti * kTile >= n_max) return; // past what this wave's tokens see (uniform over the wave)
        float s0[NB][4], s1[NB][4];
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) { st[nb].logits(t0r, s0[nb]); st[nb].logits(t1r, s1[nb]); }
        Streamer::build_v_in_place(t0r);
        Streamer::build_v_in_place(t1r);
        const bool cm0 = (ti + 1) * kTile > first_limit, cm1 = (ti + 2) * kTile > first_limit;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            float p0[4], p1[4];
            st[nb].tile_weights(ti, s0[nb], cm0, p0, nullptr);
            st[nb].tile_weights(ti + 1, s1[nb], cm1, p1, p0);
            st[nb].pv_pair(t0r, t1r, p0, p1);
        }
    };

    // ---- every thread of the workgroup runs the same rounds, two tiles and one barrier each: while the pair
    // in two of the four ring slots is computed, the next pair (fetched a round ago) goes into the other two
    // and the pair after that is requested.  A tile past the last one the workgroup sees is that tile again
    // (fetch clamps), masked out by the causal limits.
    {
        u32x4 q0 = fetch(0), q1 = fetch(1);
        park(0, q0);
        park(1, q1);
        q0 = fetch(2);
        q1 = fetch(3);
        __syncthreads();
        for (int i = 0; i < nt; i += 2) {
            park(i + 2, q0);
            park(i + 3, q1);
            q0 = fetch(i + 4);
            q1 = fetch(i + 5);
            TileRegs ta, tb;
            operands(ta, i);
            operands(tb, i + 1);
            compute_pair(ta, tb, i);
            __syncthreads();
        }
    }
    if (!has_tokens) return;

    // ---- normalise and store: a lane holds channels 8r .. 8r+7 of columns 4g .. 4g+3; the
    // denominator of column c is complete in lane c once the four lane-partials are added
    typedef __attribute__((address_space(1))) u32x4 *g_u32x4p;
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        float l = st[nb].l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int col = 4 * g + v;
            const float inv = 1.f / __shfl(l, col);
            const int t = t0 + nb * a.qpb + col / G;
            if (col / G < a.qpb && t <= tl) {
                const u32x4 o = {pack_bf16x2(st[nb].oacc[0][v] * inv, st[nb].oacc[1][v] * inv),
                                 pack_bf16x2(st[nb].oacc[2][v] * inv, st[nb].oacc[3][v] * inv),
                                 pack_bf16x2(st[nb].oacc[4][v] * inv, st[nb].oacc[5][v] * inv),
                                 pack_bf16x2(st[nb].oacc[6][v] * inv, st[nb].oacc[7][v] * inv)};
                *(g_u32x4p)(a.out + (((size_t)t * units + u) * G + col % G) * D + 8 * r) = o;
            }
        }
    }
}

int fill_tokens_per_pass(int G) { return 4 * (16 / G); }

hipError_t launch_fill_bulk(const Plan &p, const void *q, const void *k_new, const void *v_new, void *out, int n0,
                            int Tb, hipStream_t s)
{
    FillArgs a;
    a.Kc = (uint16_t *)p.k_cache; a.Vc = (uint16_t *)p.v_cache;
    a.lu = p.lu;
    a.q = (const uint16_t *)q; a.k_new = (const uint16_t *)k_new; a.v_new = (const uint16_t *)v_new;
    a.out = (uint16_t *)out;
    a.n0 = n0; a.Tb = Tb; a.N = p.N; a.G = p.G; a.units = p.units; a.lu_stride = p.ntiles * kTile;
    a.qpb = 16 / p.G;
    a.scale_log2 = 1.4426950408889634f / sqrtf(128.f);
    const long long rows = (long long)Tb * p.units;
    long long blocks = (rows + 15) / 16;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(fill_insert_kernel, dim3((unsigned)blocks), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int NB = 3, NWV = 8;
    const int QW = NWV * NB * a.qpb; // tokens per workgroup
    const long long wgs = (long long)((Tb + QW - 1) / QW) * p.units;
    hipLaunchKernelGGL((fill_attend_kernel<NB, NWV>), dim3((unsigned)wgs), dim3(64 * NWV), 0, s, a);
    return hipGetLastError();
}

} // namespace lf
