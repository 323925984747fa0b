// Fill phase in bulk (bf16, head_dim 128): the next T tokens of a cache that still has room.
//
// While a cache is filling nothing is evicted, so consecutive decode steps depend on each
// other only through the rows they append: token t attends to the rows present after its
// own insert (Sec. 2.1).  All rows are therefore written first, and the queries then go
// through attention several at a time, each column of the S^T = K Q^T product carrying one
// (token, head) pair with its own causal row limit.  A 16-column product holds floor(16 / G)
// tokens, a wave takes NB = 2 such products through every tile it loads, and the eight waves of
// a workgroup walk the same tiles for eight different sets of tokens: HBM delivers the cache
// once per 16 * floor(16 / G) tokens
// instead of once per token, and the kernel is bound by arithmetic, not by memory.  Being so, it
// loads K in the natural operand layout (half the matrix instructions for the logits).
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

// One workgroup = one (unit, group of NWV * NB * qpb consecutive tokens).  Each of its NWV waves
// owns NB * qpb of those tokens outright and streams every tile of the rows they see: the waves
// read the same K/V lines at about the same time, so the cache hierarchy serves all but one of
// the reads and HBM sees the rows once per NWV * NB * qpb tokens (32 at G = 7), while no wave ever
// has to merge with another -- there is no LDS traffic and no barrier in this kernel.  NB = 2
// products per wave leave room for two waves per SIMD, which hide each other's matrix and LDS-free
// softmax latencies better than one wave with four products does (measured 5 % / 22 % faster on
// 8192- / 4096-slot caches).
template <int NB, int NWV>
__global__ __launch_bounds__(64 * NWV) void fill_attend_kernel(const FillArgs a)
{
    constexpr int D = 128;
    // causal columns, natural K layout; the weights enter the P V product as single bf16 values (the
    // matrix pipe is not idle here as it is in the decode step, and the second product for the
    // low parts costs 8 % of the kernel): an output can differ from the decode step's by one unit in
    // the last place of bf16
    typedef MfmaStreamer<1, false, kStashNone, false, true, false, true> Streamer;
    const int G = a.G, units = a.units, QW = NB * a.qpb;
    const int ngroups = (a.Tb + NWV * QW - 1) / (NWV * QW);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, r = lane & 15;
    // late tokens see the most rows: their groups go first
    const int qg = ngroups - 1 - (int)(blockIdx.x / units), u = blockIdx.x % units;
    const int t0 = (qg * NWV + wave) * QW;
    if (t0 >= a.Tb) return; // the last group may be short of waves
    const int tl = min(t0 + QW, a.Tb) - 1;
    const int n_max = a.n0 + tl + 1;
    const int qi = r / G, h_of_r = r % G;

    Streamer st[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        const int t = t0 + nb * a.qpb + qi;
        const bool used = qi < a.qpb && t <= tl;
        st[nb].init_column(used ? (g_cu16p)(a.q + (((size_t)t * units + u) * G + h_of_r) * D) : (g_cu16p) nullptr, a.n0 + t + 1, lane, a.scale_log2);
        st[nb].Ku = (g_cu16p)(a.Kc + (size_t)u * a.N * D);
        st[nb].Vu = (g_cu16p)(a.Vc + (size_t)u * a.N * D);
        st[nb].start = 0;
        st[nb].end = n_max;
    }

    // ---- stream every tile of rows [0, n_max); two register tiles rotate
    {
        const int nfull = n_max / kTile;
        TileRegs ta, tb;
        // Per tile the V operands are built once for all the wave's products, and the causal test is
        // skipped on tiles that every one of the wave's tokens sees whole (all but the last few): both
        // come out of the vector-instruction budget that bounds this kernel.
        const int first_limit = a.n0 + t0 + 1; // rows the wave's first token sees; later tokens see more
        auto compute = [&](TileRegs &t, int ti) __attribute__((always_inline)) {
            Streamer::build_v_in_place(t);
            const bool cmask_now = (ti + 1) * kTile > first_limit;
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) st[nb].template compute_core<false, true, true>(t, ti, cmask_now);
        };
        if (nfull >= 2) {
            st[0].template load_tile<false>(ta, 0);
            st[0].template load_tile<false>(tb, 1);
            int i = 0;
            for (; i + 3 < nfull; i += 2) {
                compute(ta, i);
                st[0].template load_tile<false>(ta, i + 2);
                compute(tb, i + 1);
                st[0].template load_tile<false>(tb, i + 3);
            }
            compute(ta, i);
            if (i + 2 < nfull) st[0].template load_tile<false>(ta, i + 2);
            compute(tb, i + 1);
            if (i + 2 < nfull) compute(ta, i + 2);
        } else if (nfull == 1) {
            st[0].template load_tile<false>(ta, 0);
            compute(ta, 0);
        }
        if (n_max % kTile != 0) {
            st[0].template load_tile<true>(ta, nfull);
            st[0].template zero_ragged<true>(ta, nfull);
            Streamer::build_v_in_place(ta);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) st[nb].template compute_core<true, true, true>(ta, nfull);
        }
    }

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
    constexpr int NB = 2, NWV = 8;
    const int QW = NWV * NB * a.qpb; // tokens per workgroup
    const long long wgs = (long long)((Tb + QW - 1) / QW) * p.units;
    hipLaunchKernelGGL((fill_attend_kernel<NB, NWV>), dim3((unsigned)wgs), dim3(64 * NWV), 0, s, a);
    return hipGetLastError();
}

} // namespace lf
