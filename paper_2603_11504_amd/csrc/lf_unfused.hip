// Unfused comparison path: importance = accumulated attention weights (bf16, head_dim 128).
//
// The paper measures its fused kernel against H2O with both evicting one token after each
// attention computation (Fig. 1), describes H2O as ranking tokens by accumulated attention
// scores (Sec. 4.1) that it keeps as auxiliary per-token metadata (Sec. 2.2), and names the
// cost of such designs: importance is evaluated outside the attention kernel, re-deriving
// intermediates that kernel already had (Sec. 2.2, the paragraph on compatibility with fused kernels).
// This file is that structure with every stage written as well as the fused path's own:
//
//   1. insert      K[slot], V[slot] <- k_t, v_t; acc[slot] <- 0             (Fig. 2 left)
//   2. attention   the plain decode-attention kernel (no by-products)        (eq. 1)
//   3. accumulate  a second pass over K: alpha_h,i = 2^(t_h,i - m_h) / l_h from the
//                  attention kernel's softmax state, acc[i] += sum_h alpha_h,i, and the
//                  lowest accumulator of each workgroup's span
//   4. decide      lowest accumulator of the unit (lowest slot among equals) -> pending
//
// Steps 1, 3 and 4 live here; step 2 is the attention-only instance of the kernels the
// fused path uses.  What the comparison measures is therefore the structure alone: K is
// streamed twice, a per-slot side buffer is read and written every step, and a step is four
// launches instead of one.
#include <climits>

#include "lf_mfma_stream.h"

namespace lf {

struct UnfusedArgs {
    const uint16_t *Kc;
    uint16_t *Kw, *Vw;
    const uint16_t *q, *k_new, *v_new;
    const float *fin_m, *fin_l;
    float *acc;       // [units][NP], position order inside each 16-slot tile (pos_of_slot)
    float *part_v;    // [units][CA]
    int32_t *part_i;  // [units][CA]
    int32_t *pending, *evict_idx;
    int n, N, NP, G, LA, CA, units;
    float scale_log2;
};

__global__ __launch_bounds__(64) void unfused_insert_kernel(const UnfusedArgs a)
{
    const int u = blockIdx.x, lane = threadIdx.x;
    const int slot = a.pending[u];
    if (slot < 0 || slot >= a.N) return; // never set by this library; keeps a stray value harmless
    const size_t row = ((size_t)u * a.N + slot) * 128;
    if (lane < 16) {
        *(u32x4 *)(a.Kw + row + 8 * lane) = *(const u32x4 *)(a.k_new + (size_t)u * 128 + 8 * lane);
    } else if (lane < 32) {
        const int j = lane - 16;
        *(u32x4 *)(a.Vw + row + 8 * j) = *(const u32x4 *)(a.v_new + (size_t)u * 128 + 8 * j);
    } else if (lane == 32) {
        a.acc[(size_t)u * a.NP + (slot & ~15) + pos_of_slot(slot & 15)] = 0.f; // the slot's history starts over
    }
}

// (value, slot) pairs ordered by value, then slot
__device__ __forceinline__ void take_lower(float &bv, int &bi, float v, int i)
{
    if (v < bv || (v == bv && i < bi)) { bv = v; bi = i; }
}

struct KTile {
    u32x4 k[2][2]; // as TileRegs::k
    f32x4 a;       // accumulators of the lane's four slots (positions 4g .. 4g + 3)
};

// One workgroup = one (unit, span of LA slots); a wave takes every fourth 16-slot tile.
// K rows arrive in the operand layout of the fused kernel's S^T = K Q^T product (see
// lf_mfma_stream.h).
__global__ __launch_bounds__(256) void unfused_accumulate_kernel(const UnfusedArgs a)
{
    const int u = blockIdx.x / a.CA, c = blockIdx.x % a.CA;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, r = lane & 15;
    const int G = a.G;
    const int start = c * a.LA, end = min(start + a.LA, a.n);
    float best_v = INFINITY;
    int best_i = INT_MAX;

    if (start < end) {
        u32x4 qreg[2][2];
#pragma unroll
        for (int L = 0; L < 2; ++L)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                qreg[L][b] = u32x4{0u, 0u, 0u, 0u};
                if (r < G) qreg[L][b] = *(const u32x4 *)(a.q + ((size_t)u * G + r) * 128 + 64 * L + 8 * (2 * g + b));
            }
        const float M = (r < G) ? a.fin_m[(size_t)u * G + r] : 0.f;
        const float invL = (r < G) ? 1.f / a.fin_l[(size_t)u * G + r] : 0.f;
        const uint16_t *Ku = a.Kc + (size_t)u * a.N * 128;
        float *acc_u = a.acc + (size_t)u * a.NP;
        const int nt = (end - start + kTile - 1) / kTile;
        const int last = end - 1;
        const int n_my = (nt > wave) ? (nt - wave + 3) / 4 : 0;

        auto load = [&](KTile &t, int i) {
            const int base = start + (wave + 4 * i) * kTile;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int krow = min(base + 8 * h + (r >> 1), last);
#pragma unroll
                for (int L = 0; L < 2; ++L)
                    t.k[h][L] = __builtin_nontemporal_load(
                        (const u32x4 *)(Ku + (size_t)krow * 128 + 64 * L + 8 * (2 * g + (r & 1))));
            }
            t.a = *(const f32x4 *)(acc_u + base + 4 * g); // inside the padded row
        };
        auto consume = [&](KTile &t, int i) {
            const int base = start + (wave + 4 * i) * kTile;
            f32x4 upd;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int L = 0; L < 2; ++L) {
                    const bf16x8 ka = __builtin_bit_cast(bf16x8, t.k[h][L]);
                    d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, __builtin_bit_cast(bf16x8, qreg[L][0]), d0, 0, 0, 0);
                    d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, __builtin_bit_cast(bf16x8, qreg[L][1]), d1, 0, 0, 0);
                }
                // logits of head r at slots base + 8h + 2g and + 1 (accumulator rows 4g + v)
                const float s0 = d0[0] + d1[1], s1 = d0[2] + d1[3];
                const int slot0 = base + 8 * h + 2 * g;
                float w0 = fast_exp2(fmaf(s0, a.scale_log2, -M)) * invL; // eq. 1
                float w1 = fast_exp2(fmaf(s1, a.scale_log2, -M)) * invL;
                if (r >= G || slot0 >= end) w0 = 0.f;
                if (r >= G || slot0 + 1 >= end) w1 = 0.f;
                upd[2 * h] = t.a[2 * h] + row16_sum(w0); // summed over the group's heads
                upd[2 * h + 1] = t.a[2 * h + 1] + row16_sum(w1);
                if (r == 0) {
                    if (slot0 < end) take_lower(best_v, best_i, upd[2 * h], slot0);
                    if (slot0 + 1 < end) take_lower(best_v, best_i, upd[2 * h + 1], slot0 + 1);
                }
            }
            // four lanes write the tile's 64 bytes of accumulators with one instruction
            if (r == 0) *(f32x4 *)(acc_u + base + 4 * g) = upd;
        };

        // Two register tiles rotate; the steady-state body has no branch between a load and
        // its use, so every wait covers the older tile only.  Few registers, many waves: the
        // loads in flight come from occupancy rather than from a deep per-wave pipeline.
        KTile ta, tb;
        if (n_my >= 2) {
            load(ta, 0);
            load(tb, 1);
            int i = 0;
            for (; i + 3 < n_my; i += 2) {
                consume(ta, i);
                load(ta, i + 2);
                consume(tb, i + 1);
                load(tb, i + 3);
            }
            // 2 or 3 tiles remain; the first two are on their way
            consume(ta, i);
            if (i + 2 < n_my) load(ta, i + 2);
            consume(tb, i + 1);
            if (i + 2 < n_my) consume(ta, i + 2);
        } else if (n_my == 1) {
            load(ta, 0);
            consume(ta, 0);
        }
    }

    // ---- lowest (value, slot) of the span
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const float ov = __shfl_xor(best_v, off);
        const int oi = __shfl_xor(best_i, off);
        take_lower(best_v, best_i, ov, oi);
    }
    __shared__ float sv[4];
    __shared__ int si[4];
    if (lane == 0) { sv[wave] = best_v; si[wave] = best_i; }
    __syncthreads();
    if (tid == 0) {
        for (int w = 1; w < 4; ++w) take_lower(best_v, best_i, sv[w], si[w]);
        a.part_v[(size_t)u * a.CA + c] = best_v;
        a.part_i[(size_t)u * a.CA + c] = best_i;
    }
}

// One wave per unit: the slot the next token will cover.
__global__ __launch_bounds__(256) void unfused_decide_kernel(const UnfusedArgs a)
{
    const int lane = threadIdx.x & 63;
    const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (u >= a.units) return;
    int next = a.n; // still filling: the next free slot
    if (a.n >= a.N) {
        float bv = INFINITY;
        int bi = INT_MAX;
        for (int c = lane; c < a.CA; c += 64) take_lower(bv, bi, a.part_v[(size_t)u * a.CA + c], a.part_i[(size_t)u * a.CA + c]);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const float ov = __shfl_xor(bv, off);
            const int oi = __shfl_xor(bi, off);
            take_lower(bv, bi, ov, oi);
        }
        next = bi;
    }
    if (lane == 0) {
        a.pending[u] = next;
        if (a.evict_idx) a.evict_idx[u] = next;
    }
}

// The books in slot order: float [units][N].
__global__ __launch_bounds__(256) void unfused_scores_kernel(const float *__restrict__ acc, float *__restrict__ scores,
                                                             int N, int NP, long long total)
{
    const long long idx = (long long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= total) return;
    const long long u = idx / N;
    const int slot = (int)(idx % N);
    scores[idx] = acc[u * NP + (slot & ~15) + pos_of_slot(slot & 15)];
}

hipError_t launch_unfused_scores(const Plan &p, float *scores, hipStream_t s)
{
    const long long total = (long long)p.units * p.N;
    hipLaunchKernelGGL(unfused_scores_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p.acc, scores, p.N,
                       p.ntiles * kTile, total);
    return hipGetLastError();
}

void unfused_geometry(int units, int N, int *LA, int *CA)
{
    // spans of at most 1024 slots, shorter while the grid would not fill the chip
    int la = 1024;
    while (la > 128 && (long long)units * ((N + la - 1) / la) < 1024) la /= 2;
    *LA = la;
    *CA = (N + la - 1) / la;
}

hipError_t launch_unfused_step(const Plan &p, const StepIo &io, int n, hipStream_t s)
{
    UnfusedArgs a;
    a.Kc = (const uint16_t *)p.k_cache;
    a.Kw = (uint16_t *)p.k_cache;
    a.Vw = (uint16_t *)p.v_cache;
    a.q = (const uint16_t *)io.q;
    a.k_new = (const uint16_t *)io.k_new;
    a.v_new = (const uint16_t *)io.v_new;
    a.fin_m = p.fin_m;
    a.fin_l = p.fin_l;
    a.acc = p.acc;
    a.part_v = p.acc_part_v;
    a.part_i = p.acc_part_i;
    a.pending = p.pending;
    a.evict_idx = io.evict_idx;
    a.n = n; a.N = p.N; a.NP = p.ntiles * kTile; a.G = p.G; a.units = p.units;
    unfused_geometry(p.units, p.N, &a.LA, &a.CA);
    a.scale_log2 = 1.4426950408889634f / sqrtf(128.f);

    hipLaunchKernelGGL(unfused_insert_kernel, dim3(p.units), dim3(64), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // plain attention over the n valid rows; leaves each head's softmax state in fin_m / fin_l
    if (p.use_unit) {
        e = launch_unit_mfma(p, io.q, nullptr, nullptr, n, io.out, nullptr, s);
    } else {
        const StepIo att = {io.q, nullptr, nullptr, io.out, nullptr};
        e = launch_split_mfma(p, att, n, s);
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(unfused_accumulate_kernel, dim3(p.units * a.CA), dim3(256), 0, s, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(unfused_decide_kernel, dim3((p.units + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}

} // namespace lf
