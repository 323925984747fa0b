// Matrix-core streaming core shared by the split-K kernel and the unit-resident fused
// kernel (bf16, head_dim 128, wave64, gfx950).
//
// A wave streams 16-slot tiles of K and V exactly once, with 128-bit loads that land
// directly in the MFMA operand layouts (no LDS staging, no transposes through memory):
//
//   S^T = K Q^T      4 x v_mfma_f32_16x16x32_bf16   rows = 16 slots, cols = 16 (padded) heads
//   p   = 2^(t - m)  online softmax per head, fp32                        (eq. 1)
//   O  += P V        8 x v_mfma_f32_16x16x16_bf16, P as bf16 hi (+ lo) parts
//   U   = I |V|      8 x v_mfma_f32_16x16x16_bf16 with an identity A operand, then a
//                    16-lane row sum: u_i = ||v_i||_1                     (eq. 6)
//
// The S^T orientation makes the softmax output land in exactly the lane layout the PV
// product needs for its A operand, and V is loaded so that a lane holds the same 8
// channels of 4 consecutive slots: byte-permutes turn that into the B operand
// (contraction over slots) without leaving the register file.
//
// Lane naming: g = lane >> 4 (0..3), r = lane & 15.
//   logits / p      lane (g, r): head r, slots base + 4g + v, v = 0..3
//   O accumulators  lane (g, r): head 4g + v, channel 8r + dd, dd = 0..7
#pragma once
#include <type_traits>

#include "lf_device.h"
#include "lf_host.h"

namespace lf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// What a tile leaves behind for the eviction decision (screening values ~ u_i * p_h,i):
enum StashMode {
    kStashNone = 0,   // attention only
    kStashGlobal = 1, // bf16 values + per-tile reference, in device memory
    kStashLds = 2     // 8-bit log2 codes (quarter-octave steps) + per-tile reference, in LDS
};

// 8-bit code of a positive value w: round(4 * (kCodeBias - log2 w)) clamped to [0, 255].
// Decoding gives 2^(kCodeBias - code/4), within a factor 2^(1/8) of w for 0 < code < 255.
constexpr float kCodeBias = 16.f;

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

template <int NWAVES, bool HILO, int STASH>
struct MfmaStreamer {
    static constexpr int D = 128;
    // per-wave state
    u32x4 qreg[4];
    s16x4 ident;
    f32x4 oacc[8];
    float m, l;
    // geometry
    const uint16_t *Ku, *Vu;
    int start, end, G, g, r;
    float scale_log2;
    // stash sinks
    uint16_t *gs_w;   // kStashGlobal: [tile][G][16] bf16, tile counted from slot 0 of the unit
    float *gs_m;      // kStashGlobal: [tile][G]
    uint8_t *ls_code; // kStashLds: [G][code_stride] bytes
    float *ls_ref;    // kStashLds: [tile][G]
    int code_stride;

    __device__ __forceinline__ void init(const uint16_t *q_unit, int G_, int lane, float scale)
    {
        G = G_; g = lane >> 4; r = lane & 15; scale_log2 = scale;
#pragma unroll
        for (int cc = 0; cc < 4; ++cc) {
            qreg[cc] = u32x4{0u, 0u, 0u, 0u};
            if (r < G) qreg[cc] = *(const u32x4 *)(q_unit + (size_t)r * D + 32 * cc + 8 * g);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) ident[e] = (r == 4 * g + e) ? (short)0x3f80 : (short)0;
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) oacc[dd] = f32x4{0.f, 0.f, 0.f, 0.f};
        m = -INFINITY;
        l = 0.f;
    }

    __device__ __forceinline__ void load_tile(TileRegs &t, int ti) const
    {
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
    }

    // RAGGED: the tile may reach past `end`; rows loaded from the clamped address are zeroed
    template <bool RAGGED> __device__ __forceinline__ void compute_tile(TileRegs &t, int ti)
    {
        const int base = start + ti * kTile;
        if (RAGGED) {
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
        float tv[4];
#pragma unroll
        for (int v = 0; v < 4; ++v)
            tv[v] = (!RAGGED || base + 4 * g + v < end) ? s[v] * scale_log2 : -INFINITY;
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
        float lg[4], p[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            lg[v] = tv[v] - m; // log2 of p
            p[v] = fast_exp2(lg[v]);
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
            if (STASH != kStashNone) {
                const s16x4 va = __builtin_bit_cast(s16x4, u32x2{v01 & 0x7fff7fffu, v23 & 0x7fff7fffu});
                uacc = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(ident, va, uacc, 0, 0, 0);
            }
        }
        if (STASH == kStashGlobal) {
            // uacc[v] = partial ||v||_1 of slot 4g+v over channels {8r+dd}; sum the row's 16 lanes
            float w[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) w[v] = row16_sum(uacc[v]) * p[v];
            if (r < G) {
                const size_t rec = (size_t)(base / kTile) * G + r;
                *(u32x2 *)(gs_w + rec * kTile + 4 * g) = u32x2{pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3])};
                if (g == 0) gs_m[rec] = m;
            }
        }
        if (STASH == kStashLds) {
            uint32_t code = 0;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float lw = __builtin_amdgcn_logf(row16_sum(uacc[v])) + lg[v]; // log2(u * p)
                const float c = fminf(fmaxf(rintf(4.f * (kCodeBias - lw)), 0.f), 255.f); // NaN -> 255 side irrelevant
                code |= (uint32_t)c << (8 * v);
            }
            if (r < G) {
                *(uint32_t *)(ls_code + (size_t)r * code_stride + base + 4 * g) = code;
                if (g == 0) ls_ref[(base / kTile) * G + r] = m;
            }
        }
    }

    // Stream this wave's share of [start, end): wave w owns tiles w, w + NWAVES, ...
    // Two tiles are in flight while a third is consumed; the steady-state body has no
    // branch between a load and its use, so each wait leaves the younger loads in flight.
    __device__ __forceinline__ void run(int wave)
    {
        const int nfull = (end - start) / kTile;
        const bool ragged = (end - start) % kTile != 0;
        const int n_my = (nfull > wave) ? (nfull - wave + NWAVES - 1) / NWAVES : 0;
        TileRegs ta, tb;
        if (n_my >= 2) {
            load_tile(ta, wave);
            load_tile(tb, wave + NWAVES);
            int i = 0;
            for (; i + 3 < n_my; i += 2) {
                compute_tile<false>(ta, wave + NWAVES * i);
                load_tile(ta, wave + NWAVES * (i + 2));
                compute_tile<false>(tb, wave + NWAVES * (i + 1));
                load_tile(tb, wave + NWAVES * (i + 3));
            }
            compute_tile<false>(ta, wave + NWAVES * i);
            if (i + 2 < n_my) load_tile(ta, wave + NWAVES * (i + 2));
            compute_tile<false>(tb, wave + NWAVES * (i + 1));
            if (i + 2 < n_my) compute_tile<false>(ta, wave + NWAVES * (i + 2));
        } else if (n_my == 1) {
            load_tile(ta, wave);
            compute_tile<false>(ta, wave);
        }
        if (ragged && wave == nfull % NWAVES) {
            load_tile(ta, nfull);
            compute_tile<true>(ta, nfull);
        }
    }
};

} // namespace lf
