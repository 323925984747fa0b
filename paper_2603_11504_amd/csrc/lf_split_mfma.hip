// Split-K decode attention + score by-products on the matrix cores (bf16, head_dim 128):
// one workgroup = one (unit, split); used when there are too few (batch, KV head) units
// to give every compute unit a whole one.  Writes the split's partial softmax state and
// the bf16 screening stash to device memory; the finish kernel merges and decides.
#include "lf_mfma_stream.h"
#include "lf_split_tail.h"

namespace lf {

template <bool HILO, int STASH, bool MASKED>
__global__ __launch_bounds__(256, 2) void split_mfma_kernel(const SplitTailArgs<bf16_t> ta_in, float scale_log2,
                                                             const SplitGroup gr)
{
    constexpr int D = 128;
    SplitTailArgs<bf16_t> ta = ta_in;
    const int blk = split_group_select(ta, gr);
    const int n = ta.n, N = ta.N, G = ta.G, L = ta.L, C = ta.C, ntiles = ta.ntiles, c_active = ta.c_active;
    const uint16_t *Kc = (const uint16_t *)ta.Kc, *Vc = (const uint16_t *)ta.Vc, *q = (const uint16_t *)ta.q;
    float *part_m = ta.part_m, *part_l = ta.part_l, *part_o = ta.part_o;
    uint16_t *stash_w = ta.stash_w;
    float *stash_m = ta.stash_m;
    const float *lu = ta.lu;
    const int u = blk / c_active, c = blk % c_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    split_head_insert<bf16_t, D>(ta, u, c);

    MfmaStreamer<4, HILO, STASH, MASKED> st;
    st.init((g_cu16p)(q + (size_t)u * G * D), G, lane, scale_log2);
    st.Ku = (g_cu16p)(Kc + (size_t)u * N * D);
    st.Vu = (g_cu16p)(Vc + (size_t)u * N * D);
    st.start = c * L;
    st.end = min(c * L + L, n);
    st.gs_w = (g_u16p)(stash_w + (size_t)u * ntiles * G * kTile); // tile records count from slot 0 of the unit
    st.gs_m = (g_f32p)(stash_m + (size_t)u * ntiles * G);
    st.lu_unit = (g_cf32p)(lu + (size_t)u * ntiles * kTile);
    st.run(wave);

    // ---- merge the 4 waves through LDS, write the split's partial state
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ __align__(16) float sm_o[4][16][D + 4];
    const int g = lane >> 4, r = lane & 15;
    float l = st.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (g == 0) { sm_m[wave][r] = st.m; sm_l[wave][r] = l; }
    // a lane holds channels 8r .. 8r+7 of heads 4g .. 4g+3: two 16-byte stores per head
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        float *row = &sm_o[wave][4 * g + v][8 * r];
        *(f32x4 *)row = f32x4{st.oacc[0][v], st.oacc[1][v], st.oacc[2][v], st.oacc[3][v]};
        *(f32x4 *)(row + 4) = f32x4{st.oacc[4][v], st.oacc[5][v], st.oacc[6][v], st.oacc[7][v]};
    }
    __syncthreads();
    const size_t pbase = ((size_t)u * C + c) * G;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int h = idx / D, d = idx % D;
        const float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
        float acc = 0.f, lacc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = merge_weight(sm_m[w][h], M);
            acc += a * sm_o[w][h][d];
            lacc += a * sm_l[w][h];
        }
        part_o[(pbase + h) * D + d] = acc;
        if (d == 0) { part_m[pbase + h] = M; part_l[pbase + h] = lacc; }
    }
    split_tail<bf16_t, D>(ta, u);
}

hipError_t launch_split_mfma(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    const SplitTailArgs<bf16_t> ta = make_tail_args<bf16_t>(p, io, n, n_caches);
    const SplitGroup gr = make_split_group(p, table, p.units * ta.c_active);
    const float scale_log2 = 1.4426950408889634f / sqrtf(128.f);
    const dim3 grid(p.units * ta.c_active * n_caches);
    if (p.flags & 1u)
        hipLaunchKernelGGL((split_mfma_kernel<true, kStashNone, false>), grid, dim3(256), 0, s, ta, scale_log2, gr);
    else if (p.masked)
        hipLaunchKernelGGL((split_mfma_kernel<true, kStashGlobal, true>), grid, dim3(256), 0, s, ta, scale_log2, gr);
    else
        hipLaunchKernelGGL((split_mfma_kernel<true, kStashGlobal, false>), grid, dim3(256), 0, s, ta, scale_log2, gr);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !ta.fused_tail && ta.c_active > 1) e = launch_split_finish<bf16_t, 128>(ta, p.units, gr, n_caches, s);
    return e;
}

} // namespace lf
