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

constexpr int kMaxCand = 256; // candidates listed in LDS; more than this falls back to a slow scan

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
__device__ double exact_score_bf16(const uint16_t *__restrict__ krow, const uint16_t *__restrict__ vrow,
                                   const float (*qs)[128], int G, const float *sM, const float *sL, int lane)
{
    const int h = lane >> 2, part = lane & 3;
    // ||v||_1: two channels per lane, summed over the wave
    const uint32_t vv = *(const uint32_t *)(vrow + 2 * lane);
    double l1 = fabs((double)bf16_lo(vv)) + fabs((double)bf16_hi(vv));
    l1 = wave_sum_f64(l1);
    // q_h . k over this lane's 32 channels
    double dot = 0.0;
    if (h < G) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const u32x4 kk = *(const u32x4 *)(krow + 32 * part + 8 * c);
            const f32x4 qa = *(const f32x4 *)(&qs[h][32 * part + 8 * c]);
            const f32x4 qb = *(const f32x4 *)(&qs[h][32 * part + 8 * c + 4]);
            dot = fma((double)qa[0], (double)bf16_lo(kk.x), dot);
            dot = fma((double)qa[1], (double)bf16_hi(kk.x), dot);
            dot = fma((double)qa[2], (double)bf16_lo(kk.y), dot);
            dot = fma((double)qa[3], (double)bf16_hi(kk.y), dot);
            dot = fma((double)qb[0], (double)bf16_lo(kk.z), dot);
            dot = fma((double)qb[1], (double)bf16_hi(kk.z), dot);
            dot = fma((double)qb[2], (double)bf16_lo(kk.w), dot);
            dot = fma((double)qb[3], (double)bf16_hi(kk.w), dot);
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

template <bool HILO, int STASH>
__global__ __launch_bounds__(512, 1) void unit_mfma_kernel(
    uint16_t *__restrict__ Kc, uint16_t *__restrict__ Vc, const uint16_t *__restrict__ q,
    const uint16_t *__restrict__ k_new, const uint16_t *__restrict__ v_new, int n, int N, int G,
    int code_stride, int ntiles, int32_t *__restrict__ pending, uint16_t *__restrict__ out,
    int32_t *__restrict__ evict_idx, float *__restrict__ fin_m, float *__restrict__ fin_l,
    uint16_t *__restrict__ q_last, float *__restrict__ lu, float scale_log2)
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
    __shared__ float qs[16][D];            // the query as floats, for the exact re-scoring
    __shared__ int cand_list[kMaxCand];
    __shared__ int cand_count;

    const int u = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    uint16_t *Ku = Kc + (size_t)u * N * D;
    uint16_t *Vu = Vc + (size_t)u * N * D;
    const uint16_t *qu = q + (size_t)u * G * D;
    float *lu_u = lu + (size_t)u * ntiles * kTile;

    // ---- insert (Fig. 2 left): done by the wave that will stream that tile, so that its
    // own later loads of the row are ordered behind the stores
    if (STASH != kStashNone) {
        const int slot = pending[u];
        if (slot >= 0 && slot < N && ((slot / kTile) % NW) == wave) {
            if (lane < 16)
                *(u32x4 *)(Ku + (size_t)slot * D + 8 * lane) = *(const u32x4 *)(k_new + (size_t)u * D + 8 * lane);
            // every 16-lane row sums |v_new| redundantly; rows 1 stores V, lane 32 the log2 norm
            const u32x4 vv = *(const u32x4 *)(v_new + (size_t)u * D + 8 * r);
            float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                       fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
            a1 = row16_sum(a1);
            if (g == 1) *(u32x4 *)(Vu + (size_t)slot * D + 8 * r) = vv;
            if (lane == 32) lu_u[(slot & ~15) + pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
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
    st.lu_unit = lu_u;
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
    if (STASH == kStashLds) {
        for (int i = tid; i < G * D; i += 512) qs[i / D][i % D] = bf16_lo((uint32_t)qu[i]);
        if (tid == 0) cand_count = 0;
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
            // Decode every (head, slot) code once.  A decoded term is within 2^(+-1/8) of the
            // true one; code 0 has no upper bound, code 255 no lower bound.  Each thread keeps
            // the lower-bound sums of its slots in registers, the block finds the smallest
            // upper bound, and a slot can be the true minimum only if
            //   2^(-1/8) * lb_sum <= 2^(1/8) * min ub_sum.
            const int items = 4 * nt; // 4 positions each, whole tiles
            constexpr int kRegIters = 8; // 512 threads x 4 positions x 8 = 16384 slots held in registers
            const int iters = (items + 511) / 512;
            auto decode_item = [&](int item, float *ub4, float *lb4) {
                const int tile = item >> 2;
#pragma unroll
                for (int e = 0; e < 4; ++e) ub4[e] = lb4[e] = 0.f;
                for (int h = 0; h < G; ++h) {
                    const uint32_t c4 = *(const uint32_t *)(ls_code + (size_t)h * code_stride + 4 * item);
                    const float f = ls_ref[tile * G + h];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const uint32_t c = (c4 >> (8 * e)) & 255u;
                        const float d = fast_exp2(-0.25f * (float)c) * f;
                        ub4[e] += (c == 0u) ? INFINITY : d;
                        lb4[e] += (c == 255u) ? 0.f : d;
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
            if (iters <= kRegIters) {
                float lbs[kRegIters][4];
#pragma unroll
                for (int it = 0; it < kRegIters; ++it) {
                    const int item = it * 512 + tid;
#pragma unroll
                    for (int e = 0; e < 4; ++e) lbs[it][e] = INFINITY;
                    if (it < iters && item < items) {
                        float ub4[4];
                        decode_item(item, ub4, lbs[it]);
                        ub_min = fminf(ub_min, fminf(fminf(ub4[0], ub4[1]), fminf(ub4[2], ub4[3])));
                    }
                }
                const float thr = block_min(ub_min) * 1.1893f * 1.0001f;
#pragma unroll
                for (int it = 0; it < kRegIters; ++it)
                    if (it < iters) list_candidates(it * 512 + tid, lbs[it], thr);
            } else { // budgets beyond the register window: decode twice
                for (int it = 0; it < iters; ++it) {
                    const int item = it * 512 + tid;
                    if (item < items) {
                        float ub4[4], lb4[4];
                        decode_item(item, ub4, lb4);
                        ub_min = fminf(ub_min, fminf(fminf(ub4[0], ub4[1]), fminf(ub4[2], ub4[3])));
                    }
                }
                const float thr = block_min(ub_min) * 1.1893f * 1.0001f;
                for (int it = 0; it < iters; ++it) {
                    const int item = it * 512 + tid;
                    if (item < items) {
                        float ub4[4], lb4[4];
                        decode_item(item, ub4, lb4);
                        list_candidates(item, lb4, thr);
                    }
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
                    const double v = exact_score_bf16(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qs, G, sM, sL, lane);
                    if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
                }
            } else {
                // far more candidates than the list holds (e.g. scores underflowing en masse):
                // every wave re-scores its share of ALL slots; slow, but still exact
                for (int cs = wave; cs < n; cs += NW) {
                    const double v = exact_score_bf16(Ku + (size_t)cs * D, Vu + (size_t)cs * D, qs, G, sM, sL, lane);
                    if (v < bv || (v == bv && cs < bi)) { bv = v; bi = cs; }
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
    size_t lds = unit_mfma_lds_bytes(p.N, p.G, stash);
    // With at most a few workgroups per compute unit, ask for more than half of the
    // CU's LDS so that no CU is handed two of them while another one idles.
    if (p.units <= 2 * 256 && lds < 81 * 1024) lds = 81 * 1024;
    const int code_stride = (p.N + 63) / 64 * 64;
    const float scale_log2 = 1.4426950408889634f / sqrtf(128.f);
    static bool attr_done[2] = {false, false};
#define LF_UNIT(STASH, IDX)                                                                          \
    do {                                                                                              \
        if (!attr_done[IDX]) {                                                                        \
            hipError_t e = hipFuncSetAttribute((const void *)unit_mfma_kernel<true, STASH>,           \
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)kUnitLdsLimit); \
            if (e != hipSuccess) return e;                                                            \
            attr_done[IDX] = true;                                                                    \
        }                                                                                             \
        hipLaunchKernelGGL((unit_mfma_kernel<true, STASH>), dim3(p.units), dim3(512), lds, s,         \
                           (uint16_t *)p.k_cache, (uint16_t *)p.v_cache, (const uint16_t *)q,         \
                           (const uint16_t *)k_new, (const uint16_t *)v_new, n, p.N, p.G, code_stride, \
                           p.ntiles, p.pending, (uint16_t *)out, evict_idx, p.fin_m, p.fin_l,         \
                           (uint16_t *)p.q_last, p.lu, scale_log2);                                         \
    } while (0)
    if (stash) LF_UNIT(kStashLds, 0); else LF_UNIT(kStashNone, 1);
#undef LF_UNIT
    return hipGetLastError();
}

} // namespace lf
