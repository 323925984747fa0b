// Split-K decode attention + score by-products on the matrix cores (bf16, head_dim 128):
// one workgroup = one (unit, split); used when there are too few (batch, KV head) units
// to give every compute unit a whole one.  Writes the split's partial softmax state and
// the bf16 screening stash to device memory; the finish kernel merges and decides.
#include "lf_mfma_stream.h"

namespace lf {

template <bool HILO, int STASH>
__global__ __launch_bounds__(256, 2) void split_mfma_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Vc, const uint16_t *__restrict__ q,
    int n, int N, int G, int L, int C, int ntiles, int c_active,
    float *__restrict__ part_m, float *__restrict__ part_l, float *__restrict__ part_o,
    uint16_t *__restrict__ stash_w, float *__restrict__ stash_m, const float *__restrict__ lu,
    float scale_log2)
{
    constexpr int D = 128;
    const int u = blockIdx.x / c_active, c = blockIdx.x % c_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    MfmaStreamer<4, HILO, STASH> st;
    st.init(q + (size_t)u * G * D, G, lane, scale_log2);
    st.Ku = Kc + (size_t)u * N * D;
    st.Vu = Vc + (size_t)u * N * D;
    st.start = c * L;
    st.end = min(c * L + L, n);
    st.gs_w = stash_w + (size_t)u * ntiles * G * kTile; // tile records count from slot 0 of the unit
    st.gs_m = stash_m + (size_t)u * ntiles * G;
    st.lu_unit = lu + (size_t)u * ntiles * kTile;
    st.run(wave);

    // ---- merge the 4 waves through LDS, write the split's partial state
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ float sm_o[4][16][D + 4];
    const int g = lane >> 4, r = lane & 15;
    float l = st.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (g == 0) { sm_m[wave][r] = st.m; sm_l[wave][r] = l; }
#pragma unroll
    for (int dd = 0; dd < 8; ++dd)
#pragma unroll
        for (int v = 0; v < 4; ++v) sm_o[wave][4 * g + v][8 * r + dd] = st.oacc[dd][v];
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
}

hipError_t launch_split_mfma(const Plan &p, const void *q, int n, hipStream_t s)
{
    const int c_active = (n + p.L - 1) / p.L;
    const float scale_log2 = 1.4426950408889634f / sqrtf(128.f);
#define LF_SPLIT(STASH)                                                                             \
    hipLaunchKernelGGL((split_mfma_kernel<true, STASH>), dim3(p.units * c_active), dim3(256), 0, s, \
                       (const uint16_t *)p.k_cache, (const uint16_t *)p.v_cache, (const uint16_t *)q, \
                       n, p.N, p.G, p.L, p.C, p.ntiles, c_active, p.part_m, p.part_l, p.part_o,    \
                       p.stash_w, p.stash_m, p.lu, scale_log2)
    if (p.flags & 1u) LF_SPLIT(kStashNone); else LF_SPLIT(kStashGlobal);
#undef LF_SPLIT
    return hipGetLastError();
}

} // namespace lf
