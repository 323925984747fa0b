// Split-K decode attention + score by-products on the matrix cores in fp32 arithmetic
// (v_mfma_f32_16x16x4_f32): fp32 caches of head_dim 64 or 128, and bf16 caches of head_dim 64
// (their elements are widened on load).  Groups of up to 16 query heads per KV head.
//
// One workgroup = one (unit, split), four waves; wave w owns tiles w, w + 4, ... of the split.
// Lane naming: g = lane >> 4, r = lane & 15.  Per 16-slot tile and wave:
//
//   S^T = K Q^T   A = K rows (row r of the tile), B = Q^T (head r): D / 4 products; the 4-wide
//                 contraction index of product (c, e) stands for channels 16 c + 4 g + e, so that a
//                 lane's operands for four products come from one 16-byte load.  The accumulator
//                 register v of lane (g, r) is the logit of (slot 4 g + v, head r).
//   p = 2^(t-m)   online softmax per head in fp32, reference raised lazily       (eq. 1)
//   O += P V      A = P (head r, slots 4 g + v: exactly what the lane holds), B = V: lane (g, r)
//                 loads channels 64 cc + 4 r .. + 3 of slots 4 g + v (16 bytes, whole lines per
//                 instruction); product (cc, e, v) contracts over the slots 4 g + v and leaves
//                 O[head 4 g + v'][channel 64 cc + 4 r + e] in accumulator register v'.
//   stash         bf16(||v_i||_1 p_h,i) per (head, slot) + the tile's reference per head, in
//                 device memory, slot order inside a tile                          (eq. 6)
//
// The weights enter P V as fp32: no splitting into parts.  ||v||_1 comes from the V rows in
// registers (a sum over the lane's channels and a DPP row sum): no side array is needed.
#include <type_traits>

#include "lf_device.h"
#include "lf_host.h"
#include "lf_split_tail.h"

namespace lf {

namespace {

constexpr float kRefSlack = 8.f;      // the reference is raised when a logit passes it by more than this (log2)
constexpr float kRefNone = -3.0e38f;  // reference of a state that has seen no valid slot yet

// four consecutive elements as floats
__device__ __forceinline__ f32x4 load4(const float *p) { return *(const f32x4 *)p; }
__device__ __forceinline__ f32x4 load4(const bf16_t *p)
{
    const u32x2 t = *(const u32x2 *)p;
    return f32x4{bf16_lo(t.x), bf16_hi(t.x), bf16_lo(t.y), bf16_hi(t.y)};
}

// A tile's K rows or its V rows: D / 16 registers of four floats either way, so the same buffer
// serves both in turn (three of them rotate, see below).
//   as K: x[c]          = row r, channels 16 c + 4 g .. + 3
//   as V: x[v * VC + cc] = row 4 g + v, channels 64 cc + 4 r .. + 3
template <int D> struct Rows32 {
    f32x4 x[D / 16];
};

} // namespace

template <typename T, int D, bool STASH>
__global__ __launch_bounds__(256) void split_mfma32_kernel(const SplitTailArgs<T> ta_in, float scale_log2, const SplitGroup gr)
{
    constexpr int KC = D / 16, VC = D / 64;
    SplitTailArgs<T> ta = ta_in;
    const int blk = split_group_select(ta, gr);
    const int n = ta.n, N = ta.N, G = ta.G, L = ta.L, C = ta.C, ntiles = ta.ntiles, c_active = ta.c_active;
    const int u = blk / c_active, c = blk % c_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, r = lane & 15;
    split_head_insert<T, D>(ta, u, c);

    const T *Ku = ta.Kc + (size_t)u * N * D;
    const T *Vu = ta.Vc + (size_t)u * N * D;
    const int start = c * L, end = min(start + L, n);
    const int nt = (end - start + kTile - 1) / kTile;
    const int last = end - 1;
    const float *lu_u = ta.masked ? ta.lu + (size_t)u * ntiles * kTile : nullptr;
    uint16_t *gs_w = ta.stash_w + (size_t)u * ntiles * G * kTile; // tile records count from slot 0 of the unit
    float *gs_m = ta.stash_m + (size_t)u * ntiles * G;

    f32x4 qr[KC];
#pragma unroll
    for (int cc = 0; cc < KC; ++cc) {
        qr[cc] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (r < G) qr[cc] = load4(ta.q + ((size_t)u * G + r) * D + 16 * cc + 4 * g);
    }
    f32x4 oacc[VC][4]; // oacc[cc][e][v]: head 4 g + v, channel 64 cc + 4 r + e
#pragma unroll
    for (int cc = 0; cc < VC; ++cc)
#pragma unroll
        for (int e = 0; e < 4; ++e) oacc[cc][e] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = kRefNone, l = 0.f; // reference (log2 domain) and lane-partial denominator of head r

    auto load_k = [&](Rows32<D> &t, int ti) __attribute__((always_inline)) {
        const int base = start + ti * kTile;
        const T *krow = Ku + (size_t)min(base + r, last) * D + 4 * g;
#pragma unroll
        for (int cc = 0; cc < KC; ++cc) t.x[cc] = load4(krow + 16 * cc);
    };
    auto load_v = [&](Rows32<D> &t, int ti) __attribute__((always_inline)) {
        const int base = start + ti * kTile;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const T *vrow = Vu + (size_t)min(base + 4 * g + v, last) * D + 4 * r;
#pragma unroll
            for (int cc = 0; cc < VC; ++cc) t.x[v * VC + cc] = load4(vrow + 64 * cc);
        }
    };
    // logits and softmax weights p[v] of (slot 4 g + v, head r)
    auto logits_softmax = [&](const Rows32<D> &t, int ti, float *p) __attribute__((always_inline)) {
        const int base = start + ti * kTile;
        // four accumulators, so that consecutive matrix instructions do not depend on each other
        f32x4 dd[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) dd[e] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < KC; ++cc)
#pragma unroll
            for (int e = 0; e < 4; ++e) dd[e] = __builtin_amdgcn_mfma_f32_16x16x4f32(t.x[cc][e], qr[cc][e], dd[e], 0, 0, 0);
        float s[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            s[v] = (dd[0][v] + dd[1][v]) + (dd[2][v] + dd[3][v]);
            if (base + 4 * g + v >= end) s[v] = -INFINITY; // past the valid rows (the row read was a clamped one)
        }
        // explicit mask (Alg. 1's M): NaN in the side array (tile position order) marks an invalid slot
        if (lu_u) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float x = lu_u[base + tail_pos_of_slot(4 * g + v)];
                if (x != x) s[v] = -INFINITY;
            }
        }
        const float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])) * scale_log2;
        if (__any(mx > m + kRefSlack)) { // rare: first tile, or a logit far above everything so far
            float mw = fmaxf(mx, __shfl_xor(mx, 16));
            mw = fmaxf(mw, __shfl_xor(mw, 32));
            const float m_new = (mw > m + kRefSlack) ? mw : m;
            const float a = fast_exp2(m - m_new);
            l *= a;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float av = __shfl(a, 4 * g + v); // factor of head 4g+v lives in lane 4g+v
#pragma unroll
                for (int cc = 0; cc < VC; ++cc)
#pragma unroll
                    for (int e = 0; e < 4; ++e) oacc[cc][e][v] *= av;
            }
            m = m_new;
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = fast_exp2(fmaf(s[v], scale_log2, -m)); // 0 for invalid slots
            l += p[v];
        }
    };
    auto output_stash = [&](const Rows32<D> &t, int ti, const float *p) __attribute__((always_inline)) {
        const int base = start + ti * kTile;
        // O += P V: product v contracts over the slots 4 g' + v
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int cc = 0; cc < VC; ++cc)
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    oacc[cc][e] = __builtin_amdgcn_mfma_f32_16x16x4f32(p[v], t.x[v * VC + cc][e], oacc[cc][e], 0, 0, 0);
        if (STASH) {
            float w[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float au = 0.f;
#pragma unroll
                for (int cc = 0; cc < VC; ++cc)
#pragma unroll
                    for (int e = 0; e < 4; ++e) au += fabsf(t.x[v * VC + cc][e]);
                w[v] = row16_sum(au) * p[v]; // ||v||_1 * p
            }
            if (r < G) {
                const size_t rec = (size_t)(base / kTile) * G + r;
                const uint32_t w01 = f32_to_bf16_bits(w[0]) | (f32_to_bf16_bits(w[1]) << 16);
                const uint32_t w23 = f32_to_bf16_bits(w[2]) | (f32_to_bf16_bits(w[3]) << 16);
                *(u32x2 *)(gs_w + rec * kTile + 4 * g) = u32x2{w01, w23};
                if (g == 0) gs_m[rec] = m;
            }
        }
    };

    // Three row buffers rotate.  While tile i's logits are formed from one, the next tile's K rows
    // are on their way into the free one and tile i's V rows sit in the third; once the logits are
    // done their buffer takes the next tile's V rows.  Loads past the wave's last tile re-read that
    // tile (never used), which keeps the loop free of branches between a load and its use.
    {
        const int n_my = (nt > wave) ? (nt - wave + 3) / 4 : 0;
        Rows32<D> ra, rb, rc;
        auto step = [&](int i, Rows32<D> &kb, Rows32<D> &vb, Rows32<D> &fb) __attribute__((always_inline)) {
            const int nxt = wave + 4 * min(i + 1, n_my - 1);
            float p[4];
            load_k(fb, nxt);
            logits_softmax(kb, wave + 4 * i, p);
            load_v(kb, nxt);
            output_stash(vb, wave + 4 * i, p);
        };
        if (n_my >= 1) {
            load_k(ra, wave);
            load_v(rb, wave);
            for (int i = 0; i < n_my; i += 3) {
                step(i, ra, rb, rc);
                if (i + 1 < n_my) step(i + 1, rc, ra, rb);
                if (i + 2 < n_my) step(i + 2, rb, rc, ra);
            }
        }
    }

    // ---- merge the 4 waves through LDS, write the split's partial state
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ __align__(16) float sm_o[4][16][D + 4];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (g == 0) { sm_m[wave][r] = (m == kRefNone) ? -INFINITY : m; sm_l[wave][r] = l; }
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int cc = 0; cc < VC; ++cc)
            *(f32x4 *)&sm_o[wave][4 * g + v][64 * cc + 4 * r] = f32x4{oacc[cc][0][v], oacc[cc][1][v], oacc[cc][2][v], oacc[cc][3][v]};
    __syncthreads();
    const size_t pbase = ((size_t)u * C + c) * G;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int h = idx / D, dch = idx % D;
        const float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
        float acc = 0.f, lacc = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float a = merge_weight(sm_m[w][h], M);
            acc += a * sm_o[w][h][dch];
            lacc += a * sm_l[w][h];
        }
        ta.part_o[(pbase + h) * D + dch] = acc;
        if (dch == 0) { ta.part_m[pbase + h] = M; ta.part_l[pbase + h] = lacc; }
    }
    split_tail<T, D>(ta, u);
}

template <typename T, int D>
static hipError_t launch_mfma32(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    const SplitTailArgs<T> ta = make_tail_args<T>(p, io, n, n_caches);
    const SplitGroup gr = make_split_group(p, table, p.units * ta.c_active);
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
    const dim3 grid(p.units * ta.c_active * n_caches);
    if (p.flags & 1u)
        hipLaunchKernelGGL((split_mfma32_kernel<T, D, false>), grid, dim3(256), 0, s, ta, scale_log2, gr);
    else
        hipLaunchKernelGGL((split_mfma32_kernel<T, D, true>), grid, dim3(256), 0, s, ta, scale_log2, gr);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !ta.fused_tail && ta.c_active > 1) e = launch_split_finish<T, D>(ta, p.units, gr, n_caches, s);
    return e;
}

hipError_t launch_split_mfma32(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    if (p.dtype == 0)
        return p.D == 64 ? launch_mfma32<float, 64>(p, io, n, s, table, n_caches) : launch_mfma32<float, 128>(p, io, n, s, table, n_caches);
    if (p.D == 64) return launch_mfma32<bf16_t, 64>(p, io, n, s, table, n_caches);
    return hipErrorInvalidValue; // bf16 with head_dim 128 has kernels of its own
}

} // namespace lf
