// Split-K decode attention + score by-products on the matrix cores (bf16, head_dim 128).
//
// One workgroup = one (unit, split) of the static cache; its 4 waves take 16-slot tiles
// round-robin and stream K and V exactly once with 128-bit loads straight into the MFMA
// operand layouts (no LDS staging, no transposes through memory):
//
//   S^T = K Q^T      4 x v_mfma_f32_16x16x32_bf16   rows = 16 slots, cols = 16 (padded) heads
//   p   = 2^(t - m)  online softmax per head, fp32                        (eq. 1)
//   O  += P V        8 x v_mfma_f32_16x16x16_bf16, P as bf16 hi (+ lo) parts
//   U   = I |V|      8 x v_mfma_f32_16x16x16_bf16 with an identity A operand, then a
//                    16-lane row sum: u_i = ||v_i||_1                     (eq. 6)
//
// The S^T orientation makes the softmax output land in exactly the lane layout the PV
// product needs for its A operand, and V is loaded so that a lane holds the same 8
// channels of 4 consecutive slots: four byte-permutes per channel pair turn that into
// the B operand (contraction over slots) without leaving the register file.
// Per tile the kernel stores bf16(u_i * p_h,i) and the reference m_h it is relative to;
// the finish kernel screens with these and settles the argmin exactly.
#include "lf_device.h"
#include "lf_host.h"

namespace lf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

struct TileRegs {
    u32x4 k[4]; // k[c]: row (lane&15) of the tile, channels 32c + 8*(lane>>4) .. +7
    u32x4 v[4]; // v[e]: row 4*(lane>>4) + e, channels 8*(lane&15) .. +7
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

template <bool HILO>
__global__ __launch_bounds__(256, 2) void split_mfma_kernel(
    const uint16_t *__restrict__ Kc, const uint16_t *__restrict__ Vc, const uint16_t *__restrict__ q,
    int n, int N, int G, int L, int C, int ntiles, int c_active,
    float *__restrict__ part_m, float *__restrict__ part_l, float *__restrict__ part_o,
    uint16_t *__restrict__ stash_w, float *__restrict__ stash_m, float scale_log2, int write_stash)
{
    constexpr int D = 128;
    const int u = blockIdx.x / c_active, c = blockIdx.x % c_active;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    const int start = c * L;
    const int end = min(start + L, n);
    const int nt = (end - start + kTile - 1) / kTile;
    const uint16_t *Ku = Kc + (size_t)u * N * D;
    const uint16_t *Vu = Vc + (size_t)u * N * D;

    // Q^T operand: lane (g, r) holds head r, channels 32c + 8g .. +7 (zero rows pad G to 16)
    u32x4 qreg[4];
#pragma unroll
    for (int cc = 0; cc < 4; ++cc) {
        qreg[cc] = u32x4{0u, 0u, 0u, 0u};
        if (r < G) qreg[cc] = *(const u32x4 *)(q + ((size_t)u * G + r) * D + 32 * cc + 8 * g);
    }
    // identity A operand of the 16x16x16 product: A[i = r][k = 4g + e] = (r == 4g + e)
    s16x4 ident;
#pragma unroll
    for (int e = 0; e < 4; ++e) ident[e] = (r == 4 * g + e) ? (short)0x3f80 : (short)0;

    f32x4 oacc[8];
#pragma unroll
    for (int dd = 0; dd < 8; ++dd) oacc[dd] = f32x4{0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;

    auto load_tile = [&](TileRegs &t, int ti) {
        const int base = start + ti * kTile;
        const int krow = min(base + r, end - 1); // clamped: never touch a row past the valid prefix
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
            t.k[cc] = __builtin_nontemporal_load((const u32x4 *)(Ku + (size_t)krow * D + 32 * cc + 8 * g));
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int vrow = min(base + 4 * g + e, end - 1);
            t.v[e] = __builtin_nontemporal_load((const u32x4 *)(Vu + (size_t)vrow * D + 8 * r));
        }
    };

    auto compute_tile = [&](TileRegs &t, int ti) {
        const int base = start + ti * kTile;
        if (base + kTile > end) { // ragged last tile (wave-uniform): clamped rows must not count
            if (base + r >= end) {
#pragma unroll
                for (int cc = 0; cc < 4; ++cc) t.k[cc] = u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + 4 * g + e >= end) t.v[e] = u32x4{0u, 0u, 0u, 0u};
        }
        // ---- S^T = K Q^T
        f32x4 s = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
            s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.k[cc]),
                                                        __builtin_bit_cast(bf16x8, qreg[cc]), s, 0, 0, 0);
        // lane (g, r): logits of slots base + 4g + v for head r
        float tv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) tv[v] = (base + 4 * g + v < end) ? s[v] * scale_log2 : -INFINITY;
        float mx = fmaxf(fmaxf(tv[0], tv[1]), fmaxf(tv[2], tv[3]));
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m, mx);
        if (__any(m_new > m)) { // rare after the first tiles: rescale the running state
            const float a = fast_exp2(m - m_new);
            l *= a;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float av = __shfl(a, 4 * g + v); // factor of head 4g+v lives in lane 4g+v
#pragma unroll
                for (int dd = 0; dd < 8; ++dd) oacc[dd][v] *= av;
            }
            m = m_new;
        }
        float p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            p[v] = fast_exp2(tv[v] - m);
            l += p[v];
        }
        s16x4 p_hi, p_lo;
        {
            const uint32_t h01 = pack_bf16x2(p[0], p[1]), h23 = pack_bf16x2(p[2], p[3]);
            p_hi = __builtin_bit_cast(s16x4, u32x2{h01, h23});
            if (HILO) {
                const uint32_t l01 = pack_bf16x2(p[0] - bf16_lo(h01), p[1] - bf16_hi(h01));
                const uint32_t l23 = pack_bf16x2(p[2] - bf16_lo(h23), p[3] - bf16_hi(h23));
                p_lo = __builtin_bit_cast(s16x4, u32x2{l01, l23});
            }
        }
        // ---- O += P V and U = I |V|, channel 8r + dd per product
        f32x4 uacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
            const int w = dd >> 1;
            const uint32_t v01 = __builtin_amdgcn_perm(t.v[1][w], t.v[0][w], sel); // slots 4g+0, 4g+1
            const uint32_t v23 = __builtin_amdgcn_perm(t.v[3][w], t.v[2][w], sel); // slots 4g+2, 4g+3
            const s16x4 vb = __builtin_bit_cast(s16x4, u32x2{v01, v23});
            oacc[dd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vb, oacc[dd], 0, 0, 0);
            if (HILO) oacc[dd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vb, oacc[dd], 0, 0, 0);
            if (write_stash) {
                const s16x4 va = __builtin_bit_cast(s16x4, u32x2{v01 & 0x7fff7fffu, v23 & 0x7fff7fffu});
                uacc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ident, va, uacc, 0, 0, 0);
            }
        }
        if (write_stash) {
            // uacc[v] = partial ||v||_1 of slot 4g+v over channels {8r+dd}; sum the 16 lanes of the row
            float w[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) w[v] = row16_sum(uacc[v]) * p[v];
            if (r < G) {
                const size_t rec = ((size_t)u * ntiles + (size_t)(base / kTile)) * G + r;
                *(u32x2 *)(stash_w + rec * kTile + 4 * g) = u32x2{pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3])};
                if (g == 0) stash_m[rec] = m;
            }
        }
    };

    // ---- software pipeline: two tiles in flight per wave
    TileRegs ta, tb;
    int ti = wave;
    if (ti < nt) load_tile(ta, ti);
    for (; ti < nt; ti += 8) {
        if (ti + 4 < nt) load_tile(tb, ti + 4);
        compute_tile(ta, ti);
        if (ti + 8 < nt) load_tile(ta, ti + 8);
        if (ti + 4 < nt) compute_tile(tb, ti + 4);
    }

    // ---- merge the 4 waves through LDS, write the split's partial state
    __shared__ float sm_m[4][16], sm_l[4][16];
    __shared__ float sm_o[4][16][D + 4];
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (g == 0) { sm_m[wave][r] = m; sm_l[wave][r] = l; }
#pragma unroll
    for (int dd = 0; dd < 8; ++dd)
#pragma unroll
        for (int v = 0; v < 4; ++v) sm_o[wave][4 * g + v][8 * r + dd] = oacc[dd][v];
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
    const int write_stash = (p.flags & 1u) ? 0 : 1;
    hipLaunchKernelGGL((split_mfma_kernel<true>), dim3(p.units * c_active), dim3(256), 0, s,
                       (const uint16_t *)p.k_cache, (const uint16_t *)p.v_cache, (const uint16_t *)q, n,
                       p.N, p.G, p.L, p.C, p.ntiles, c_active, p.part_m, p.part_l, p.part_o, p.stash_w,
                       p.stash_m, scale_log2, write_stash);
    return hipGetLastError();
}

} // namespace lf
