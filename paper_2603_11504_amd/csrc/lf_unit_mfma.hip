// Unit-resident fused decode step on the matrix cores (bf16, head_dim 128).
//
// One workgroup of 8 waves owns one (batch, KV head) unit for the whole call and does
// every step of the path in a single launch, with no intermediate in device memory:
//
//   insert   the wave that owns the pending slot's tile writes k_new / v_new into it
//   stream   all valid slots once: logits, online softmax, P V, ||v||_1     (eq. 1, eq. 6)
//            leaving an 8-bit log2 code of u_i * p_h,i per (head, slot) in LDS
//   merge    the 8 waves' softmax states -> M_h, L_h
//   evict    screen every slot with the codes (bounds within a factor 2^(1/8)), re-score
//            the few that can still be the minimum exactly in double precision, argmin
//   output   merge the 8 waves' O through LDS, normalise, round to bf16
//
// Keeping the per-slot by-products in LDS matters on this chip: even a few percent of
// HBM writes interleaved with the K/V read stream cost a quarter of the read bandwidth.
#include "lf_mfma_stream.h"

namespace lf {

__device__ __forceinline__ double wave_sum_f64(double x)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
    return x;
}

// exact LongFlowScore of one slot, computed by a whole wave in double precision (eq. 6
// with the group's heads summed); sM: reference (log2 domain), sLinv: 1 / denominator
__device__ double exact_score_bf16(const uint16_t *__restrict__ krow, const uint16_t *__restrict__ vrow,
                                   const uint16_t *__restrict__ qu, int G, const float *sM,
                                   const float *sL, int lane)
{
    const uint32_t kk = *(const uint32_t *)(krow + 2 * lane), vv = *(const uint32_t *)(vrow + 2 * lane);
    const double k0 = bf16_lo(kk), k1 = bf16_hi(kk);
    double l1 = fabs((double)bf16_lo(vv)) + fabs((double)bf16_hi(vv));
    l1 = wave_sum_f64(l1);
    const double scale_log2 = 1.4426950408889634074 / sqrt(128.0);
    double acc = 0.0;
    for (int h = 0; h < G; ++h) {
        const uint32_t qq = *(const uint32_t *)(qu + (size_t)h * 128 + 2 * lane);
        double dot = (double)bf16_lo(qq) * k0 + (double)bf16_hi(qq) * k1;
        dot = wave_sum_f64(dot);
        acc += exp2(dot * scale_log2 - (double)sM[h]) / (double)sL[h];
    }
    return acc * l1;
}

template <bool HILO, int STASH>
__global__ __launch_bounds__(512, 1) void unit_mfma_kernel(
    uint16_t *__restrict__ Kc, uint16_t *__restrict__ Vc, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new, int n, int N, int G,
    int code_stride, int ntiles, int32_t *__restrict__ pending, uint16_t *__restrict__ out,
    int32_t *__restrict__ evict_idx, float *__restrict__ fin_m, float *__restrict__ fin_l,
    uint16_t *__restrict__ q_last, float scale_log2)
{
    constexpr int D = 128, NW = 8, OPAD = D + 4;
    extern __shared__ __align__(16) unsigned char smem[];
    // LDS map: [codes G*code_stride][refs ntiles*G floats] ... later aliased by the O merge
    uint8_t *ls_code = smem;
    float *ls_ref = (float *)(smem + (size_t)G * code_stride);
    __shared__ float sm_m[NW][16], sm_l[NW][16], sM[16], sL[16];
    __shared__ float red_f[NW];
    __shared__ double best_v[NW];
    __shared__ int best_i[NW];

    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    uint16_t *Ku = Kc + (size_t)u * N * D;
    uint16_t *Vu = Vc + (size_t)u * N * D;
    const uint16_t *qu = q + (size_t)u * G * D;

    // ---- insert (Fig. 2 left): done by the wave that will stream that tile, so that its
    // own later loads of the row are ordered behind the stores
    if (STASH != kStashNone) {
        const int slot = pending[u];
        if (slot >= 0 && slot < N && ((slot / kTile) % NW) == wave) {
            if (lane < 16)
                *(u32x4 *)(Ku + (size_t)slot * D + 8 * lane) = *(const u32x4 *)(k_new + (size_t)u * D + 8 * lane);
            else if (lane < 32)
                *(u32x4 *)(Vu + (size_t)slot * D + 8 * (lane - 16)) =
                    *(const u32x4 *)(v_new + (size_t)u * D + 8 * (lane - 16));
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    }

    MfmaStreamer<NW, HILO, STASH> st;
    st.init(qu, G, lane, scale_log2);
    st.Ku = Ku;
    st.Vu = Vu;
    st.start = 0;
    st.end = n;
    st.ls_code = ls_code;
    st.ls_ref = ls_ref;
    st.code_stride = code_stride;
    st.run(wave);

    // ---- merge the softmax states of the 8 waves
    {
        float l = st.l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (g == 0) { sm_m[wave][r] = st.m; sm_l[wave][r] = l; }
    }
    __syncthreads();
    if (tid < 16) {
        float M = -INFINITY;
#pragma unroll
        for (int w = 0; w < NW; ++w) M = fmaxf(M, sm_m[w][tid]);
        float Ls = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) Ls += merge_weight(sm_m[w][tid], M) * sm_l[w][tid];
        sM[tid] = M;
        sL[tid] = Ls;
        if (tid < G) {
            fin_m[(size_t)u * G + tid] = M;
            fin_l[(size_t)u * G + tid] = Ls;
        }
    }
    __syncthreads();

    // ---- eviction decision (Sec. 3.2 last paragraph; Alg. 1 post-processing)
    if (STASH == kStashLds) {
        if (n < N) {
            if (tid == 0) {
                pending[u] = n;
                if (evict_idx) evict_idx[u] = n;
            }
        } else {
            // per (tile, head): factor that turns a decoded code into a normalised score term
            const int nt = (n + kTile - 1) / kTile;
            for (int i = tid; i < nt * G; i += 512) {
                const int h = i % G;
                ls_ref[i] = fast_exp2(kCodeBias + ls_ref[i] - sM[h]) / sL[h];
            }
            __syncthreads();
            // pass 1: upper bounds of all scores, block minimum.  A decoded term is within
            // 2^(+-1/8) of the true one; code 0 has no upper bound, code 255 no lower bound.
            const int items = (n + 3) / 4;
            const int iters = (items + 511) / 512;
            float ub_min = INFINITY;
            for (int it = 0; it < iters; ++it) {
                const int item = it * 512 + tid;
                if (item < items) {
                    const int tile = item >> 2;
                    float s4[4] = {0.f, 0.f, 0.f, 0.f};
                    for (int h = 0; h < G; ++h) {
                        const uint32_t c4 = *(const uint32_t *)(ls_code + (size_t)h * code_stride + 4 * item);
                        const float f = ls_ref[tile * G + h];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t c = (c4 >> (8 * e)) & 255u;
                            s4[e] += (c == 0u) ? INFINITY : fast_exp2(-0.25f * (float)c) * f;
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (4 * item + e < n) ub_min = fminf(ub_min, s4[e]);
                }
            }
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) ub_min = fminf(ub_min, __shfl_xor(ub_min, off));
            if (lane == 0) red_f[wave] = ub_min;
            __syncthreads();
            ub_min = red_f[0];
#pragma unroll
            for (int w = 1; w < NW; ++w) ub_min = fminf(ub_min, red_f[w]);
            // a slot can be the true minimum only if its lower bound does not exceed the
            // smallest upper bound: lb = 2^(-1/8) * dec, ub = 2^(1/8) * dec  ->  dec_i <= 2^(1/4) * dec_min
            const float thr = ub_min * 1.1893f * 1.0001f;

            // pass 2: exact double-precision scores of the candidates, wave-cooperative
            double bv = INFINITY;
            int bi = 0x7fffffff;
            for (int it = 0; it < iters; ++it) {
                const int item = it * 512 + tid;
                const int tile = item >> 2;
                float s4[4] = {INFINITY, INFINITY, INFINITY, INFINITY};
                if (item < items) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) s4[e] = 0.f;
                    for (int h = 0; h < G; ++h) {
                        const uint32_t c4 = *(const uint32_t *)(ls_code + (size_t)h * code_stride + 4 * item);
                        const float f = ls_ref[tile * G + h];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const uint32_t c = (c4 >> (8 * e)) & 255u;
                            s4[e] += (c == 255u) ? 0.f : fast_exp2(-0.25f * (float)c) * f; // lower-bound side
                        }
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int slot = 4 * item + e;
                    const bool cand = (item < items) && (slot < n) && (s4[e] <= thr);
                    unsigned long long bal = __ballot(cand);
                    while (bal) {
                        const int src = __ffsll((long long)bal) - 1;
                        bal &= bal - 1;
                        const int cs = __shfl(slot, src);
                        const double v = exact_score_bf16(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qu, G, sM, sL, lane);
                        if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
                    }
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
        __syncthreads(); // the codes are dead from here on: their LDS is reused below
    }

    // ---- merge O of the 8 waves through LDS (aliases the code area), normalise, store
    float *sm_o = (float *)smem; // [NW][16][OPAD]
    {
        float a4[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) a4[v] = merge_weight(sm_m[wave][4 * g + v], sM[4 * g + v]);
#pragma unroll
        for (int dd = 0; dd < 8; ++dd)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                sm_o[((size_t)wave * 16 + 4 * g + v) * OPAD + 8 * r + dd] = st.oacc[dd][v] * a4[v];
    }
    __syncthreads();
    for (int idx = tid; idx < G * D; idx += 512) {
        const int h = idx / D, d = idx % D;
        float acc = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) acc += sm_o[((size_t)w * 16 + h) * OPAD + d];
        out[((size_t)u * G + h) * D + d] = (uint16_t)f32_to_bf16_bits(acc / sL[h]);
        q_last[((size_t)u * G + h) * D + d] = qu[idx];
    }
}

size_t unit_mfma_lds_bytes(int N, int G, bool stash)
{
    const size_t merge = (size_t)8 * 16 * (128 + 4) * sizeof(float);
    if (!stash) return merge;
    const size_t code_stride = ((size_t)N + 63) / 64 * 64;
    const size_t ntiles = ((size_t)N + kTile - 1) / kTile;
    const size_t codes = (size_t)G * code_stride + ntiles * G * sizeof(float);
    return codes > merge ? codes : merge;
}

hipError_t launch_unit_mfma(const Plan &p, const void *q, const void *k_new, const void *v_new, int n,
                            void *out, int32_t *evict_idx, hipStream_t s)
{
    const bool stash = !(p.flags & 1u);
    const size_t lds = unit_mfma_lds_bytes(p.N, p.G, stash);
    const int code_stride = (p.N + 63) / 64 * 64;
    const float scale_log2 = 1.4426950408889634f / sqrtf(128.f);
    static bool attr_done[2] = {false, false};
#define LF_UNIT(STASH, IDX)                                                                          \
    do {                                                                                              \
        if (!attr_done[IDX]) {                                                                        \
            hipError_t e = hipFuncSetAttribute((const void *)unit_mfma_kernel<true, STASH>,           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 2048); \
            if (e != hipSuccess) return e;                                                            \
            attr_done[IDX] = true;                                                                    \
        }                                                                                             \
        hipLaunchKernelGGL((unit_mfma_kernel<true, STASH>), dim3(p.units), dim3(512), lds, s,         \
                           (uint16_t *)p.k_cache, (uint16_t *)p.v_cache, (const uint16_t *)q,         \
                           (const uint16_t *)k_new, (const uint16_t *)v_new, n, p.N, p.G, code_stride, \
                           p.ntiles, p.pending, (uint16_t *)out, evict_idx, p.fin_m, p.fin_l,         \
                           (uint16_t *)p.q_last, scale_log2);                                         \
    } while (0)
    if (stash) LF_UNIT(kStashLds, 0); else LF_UNIT(kStashNone, 1);
#undef LF_UNIT
    return hipGetLastError();
}

} // namespace lf
