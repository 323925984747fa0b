// Fill phase in bulk (bf16, head_dim 128): the next T tokens of a cache that still has room.
//
// While a cache is filling nothing is evicted, so consecutive decode steps depend on each
// other only through the rows they append: token t attends to the rows present after its
// own insert (Sec. 2.1).  All rows are therefore written first, and the queries then go
// through attention several at a time, each column of the S^T = K Q^T product carrying one
// (token, head) pair with its own causal row limit.  A 16-column product holds floor(16 / G)
// tokens, and a workgroup streams K and V once for NB such products: the cache is read
// once per NB * floor(16 / G) tokens instead of once per token.  The matrix and vector
// pipes, 13 % and 23 % busy in the single-query kernel, have the room: NB = 4 is where the
// per-tile arithmetic of a wave catches up with its share of HBM bandwidth (it costs the
// whole register file, one wave per SIMD; NB = 2 at two waves per SIMD is 25 % slower).
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

// One workgroup = one (unit, group of NB * qpb consecutive tokens); its 4 waves share the
// tiles of rows [0, n0 + last token + 1) and merge at the end.
template <int NB>
__global__ __launch_bounds__(256) void fill_attend_kernel(const FillArgs a)
{
    constexpr int D = 128;
    typedef MfmaStreamer<4, true, kStashNone, false, true> Streamer;
    const int G = a.G, units = a.units, QW = NB * a.qpb;
    const int ngroups = (a.Tb + QW - 1) / QW;
    // late tokens see the most rows: their groups go first
    const int qg = ngroups - 1 - (int)(blockIdx.x / units), u = blockIdx.x % units;
    const int t0 = qg * QW, tl = min(t0 + QW, a.Tb) - 1;
    const int n_max = a.n0 + tl + 1;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, r = lane & 15;
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

    // ---- stream: wave w owns tiles w, w + 4, ...; two register tiles rotate
    {
        const int nfull = n_max / kTile;
        const int n_my = (nfull > wave) ? (nfull - wave + 3) / 4 : 0;
        TileRegs ta, tb;
        auto compute = [&](TileRegs &t, int ti) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) st[nb].template compute_tile<false>(t, ti);
        };
        if (n_my >= 2) {
            st[0].template load_tile<false>(ta, wave);
            st[0].template load_tile<false>(tb, wave + 4);
            int i = 0;
            for (; i + 3 < n_my; i += 2) {
                compute(ta, wave + 4 * i);
                st[0].template load_tile<false>(ta, wave + 4 * (i + 2));
                compute(tb, wave + 4 * (i + 1));
                st[0].template load_tile<false>(tb, wave + 4 * (i + 3));
            }
            compute(ta, wave + 4 * i);
            if (i + 2 < n_my) st[0].template load_tile<false>(ta, wave + 4 * (i + 2));
            compute(tb, wave + 4 * (i + 1));
            if (i + 2 < n_my) compute(ta, wave + 4 * (i + 2));
        } else if (n_my == 1) {
            st[0].template load_tile<false>(ta, wave);
            compute(ta, wave);
        }
        if (n_max % kTile != 0 && wave == nfull % 4) {
            st[0].template load_tile<true>(ta, nfull);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) st[nb].template compute_tile<true>(ta, nfull);
        }
    }

    // ---- merge the 4 waves through LDS, one 16-column product at a time
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ __align__(16) float sm_o[4][16][D + 4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        float l = st[nb].l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) { sm_m[wave][r] = st[nb].m; sm_l[wave][r] = l; }
        // a lane holds channels 8r .. 8r+7 of columns 4g .. 4g+3: two 16-byte stores per column
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float *row = &sm_o[wave][4 * g + v][8 * r];
            *(f32x4 *)row = f32x4{st[nb].oacc[0][v], st[nb].oacc[1][v], st[nb].oacc[2][v], st[nb].oacc[3][v]};
            *(f32x4 *)(row + 4) = f32x4{st[nb].oacc[4][v], st[nb].oacc[5][v], st[nb].oacc[6][v], st[nb].oacc[7][v]};
        }
        __syncthreads();
        for (int idx = tid; idx < 16 * D; idx += 256) {
            const int col = idx / D, d = idx % D;
            const int t = t0 + nb * a.qpb + col / G;
            if (col / G < a.qpb && t <= tl) {
                const float M = fmaxf(fmaxf(sm_m[0][col], sm_m[1][col]), fmaxf(sm_m[2][col], sm_m[3][col]));
                float acc = 0.f, lacc = 0.f;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const float wgt = fast_exp2(sm_m[w][col] - M); // a wave that saw no row of this column: 2^(-3e38) = 0
                    acc += wgt * sm_o[w][col][d];
                    lacc += wgt * sm_l[w][col];
                }
                a.out[(((size_t)t * units + u) * G + col % G) * D + d] = (uint16_t)f32_to_bf16_bits(acc / lacc);
            }
        }
        __syncthreads();
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
    constexpr int NB = 4;
    const int QW = NB * a.qpb;
    const long long wgs = (long long)((Tb + QW - 1) / QW) * p.units;
    hipLaunchKernelGGL((fill_attend_kernel<NB>), dim3((unsigned)wgs), dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace lf
