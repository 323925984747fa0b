// Split-K decode attention + score by-products on the vector ALUs (any dtype).
//
// Serves fp32 caches and is the A/B partner of the matrix-core kernel for bf16.
// One workgroup = one (unit, split); a row of 16 lanes owns one 16-slot tile at a
// time, so that tile's softmax reference is fixed while its 16 slots are scored:
//   K phase  logits of the 16 slots for the G query heads       (eq. 1 numerator)
//   V phase  p = 2^(t - m), o += p v, u = ||v||_1               (eq. 1, eq. 6)
// and the tile's screening values bf16(u * p) go to the stash together with m.
#include <utility>

#include "lf_device.h"
#include "lf_host.h"
#include <cstring>

#include "lf_split_tail.h"

namespace lf {

template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// value held by lane JJ of each 16-lane row, seen by every lane of that row
template <int JJ> __device__ __forceinline__ float row16_bcast(float x)
{
    return dpp_f32<0x150 + JJ>(x); // row_newbcast:JJ
}

template <typename T, int D, int G>
__global__ __launch_bounds__(256) void split_valu_kernel(const SplitTailArgs<T> ta_in, float scale_log2, const SplitGroup gr)
{
    constexpr int EPL = D / 16; // elements per lane of a 16-lane row
    SplitTailArgs<T> ta = ta_in;
    const int blk = split_group_select(ta, gr);
    const int n = ta.n, N = ta.N, L = ta.L, C = ta.C, ntiles = ta.ntiles, c_active = ta.c_active;
    const T *Kc = ta.Kc, *Vc = ta.Vc, *q = ta.q;
    float *part_m = ta.part_m, *part_l = ta.part_l, *part_o = ta.part_o;
    uint16_t *stash_w = ta.stash_w;
    float *stash_m = ta.stash_m;
    const int write_stash = !ta.attention_only;
    const int u = blk / c_active, c = blk % c_active;
    split_head_insert<T, D>(ta, u, c);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rg = lane >> 4, j = lane & 15;
    const int start = c * L;
    const int end = min(start + L, n);
    const int nt = (end - start + kTile - 1) / kTile;
    const T *Ku = Kc + (size_t)u * N * D;
    const T *Vu = Vc + (size_t)u * N * D;

    float qf[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        RowChunk<T, EPL> r;
        r.load(q + ((size_t)u * G + h) * D + j * EPL);
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[h][e] = r.v[e];
    }
    float m[G], l[G], o[G][EPL];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        m[h] = -INFINITY;
        l[h] = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) o[h][e] = 0.f;
    }

    for (int ti = wave * 4 + rg; ti < nt; ti += 16) {
        const int base = start + ti * kTile;
        // ---- K phase: lane j ends up with the logits of slot base+j (log2 domain)
        float t[G];
#pragma unroll
        for (int h = 0; h < G; ++h) t[h] = -INFINITY;
        // explicit mask (Alg. 1's M): lane j holds the side-array entry of tile position j;
        // NaN marks an invalid slot, which is then treated like a slot past the end
        float lu_mine = 0.f;
        if (ta.masked) lu_mine = ta.lu[(size_t)u * ntiles * kTile + base + j];
        // Rows are fetched eight at a time, unconditionally (a slot past the end re-reads the
        // last valid row and is discarded afterwards): eight loads in flight per lane instead
        // of a load-wait-use chain per slot.
        const int last = end - 1;
        static_for<2>([&](auto hc) {
            constexpr int half = decltype(hc)::value;
            RowChunk<T, EPL> kr[8];
            static_for<8>([&](auto ic) {
                constexpr int jj = 8 * half + decltype(ic)::value;
                kr[jj - 8 * half].load(Ku + (size_t)min(base + jj, last) * D + j * EPL);
            });
            static_for<8>([&](auto ic) {
                constexpr int jj = 8 * half + decltype(ic)::value;
                const float lu_jj = row16_bcast<tail_pos_of_slot(jj)>(lu_mine);
                const bool valid = base + jj < end && lu_jj == lu_jj;
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    float part = 0.f;
#pragma unroll
                    for (int e = 0; e < EPL; ++e) part = fmaf(qf[h][e], kr[jj - 8 * half].v[e], part);
                    part = row16_sum(part);
                    if (jj == j) t[h] = valid ? part * scale_log2 : -INFINITY;
                }
            });
        });
        // ---- fix the tile's reference, rescale the running state once
        float p[G];
#pragma unroll
        for (int h = 0; h < G; ++h) {
            const float m_new = fmaxf(m[h], row16_max(t[h]));
            const float a = merge_weight(m[h], m_new);
            l[h] *= a;
#pragma unroll
            for (int e = 0; e < EPL; ++e) o[h][e] *= a;
            m[h] = m_new;
            p[h] = (t[h] == -INFINITY) ? 0.f : fast_exp2(t[h] - m_new);
            l[h] += p[h]; // lane-partial; summed over the row at the end
        }
        // ---- V phase
        float u_mine = 0.f;
        static_for<2>([&](auto hc) {
            constexpr int half = decltype(hc)::value;
            RowChunk<T, EPL> vr[8];
            static_for<8>([&](auto ic) {
                constexpr int jj = 8 * half + decltype(ic)::value;
                vr[jj - 8 * half].load(Vu + (size_t)min(base + jj, last) * D + j * EPL);
            });
            static_for<8>([&](auto ic) {
                constexpr int jj = 8 * half + decltype(ic)::value;
                const float lu_jj = row16_bcast<tail_pos_of_slot(jj)>(lu_mine);
                const bool valid = base + jj < end && lu_jj == lu_jj;
                RowChunk<T, EPL> &row = vr[jj - 8 * half];
                if (!valid) row.zero(); // p is 0 there, but the row itself may hold anything
                float au = 0.f;
#pragma unroll
                for (int e = 0; e < EPL; ++e) au += fabsf(row.v[e]);
                au = row16_sum(au);
                if (jj == j) u_mine = au;
#pragma unroll
                for (int h = 0; h < G; ++h) {
                    const float pj = row16_bcast<jj>(p[h]);
#pragma unroll
                    for (int e = 0; e < EPL; ++e) o[h][e] = fmaf(pj, row.v[e], o[h][e]);
                }
            });
        });
        if (write_stash) {
            const size_t rec = (size_t)u * ntiles + (size_t)(base / kTile);
#pragma unroll
            for (int h = 0; h < G; ++h) {
                stash_w[(rec * G + h) * kTile + j] = (uint16_t)f32_to_bf16_bits(u_mine * p[h]);
                if (j == 0) stash_m[rec * G + h] = m[h];
            }
        }
    }

    // ---- merge: 4 rows of a wave, then the 4 waves through LDS
    __shared__ float sm_m[4][G], sm_l[4][G], sm_o[4][G][D];
#pragma unroll
    for (int h = 0; h < G; ++h) {
        float lh = row16_sum(l[h]);
        float M = fmaxf(m[h], __shfl_xor(m[h], 16));
        M = fmaxf(M, __shfl_xor(M, 32));
        const float a = merge_weight(m[h], M);
        lh *= a;
        lh += __shfl_xor(lh, 16);
        lh += __shfl_xor(lh, 32);
#pragma unroll
        for (int e = 0; e < EPL; ++e) {
            float x = o[h][e] * a;
            x += __shfl_xor(x, 16);
            x += __shfl_xor(x, 32);
            if (rg == 0) sm_o[wave][h][j * EPL + e] = x;
        }
        if (lane == 0) { sm_m[wave][h] = M; sm_l[wave][h] = lh; }
    }
    __syncthreads();
    const size_t pbase = ((size_t)u * C + c) * G;
    for (int idx = tid; idx < G * D; idx += 256) {
        const int h = idx / D, d = idx % D;
        float M = fmaxf(fmaxf(sm_m[0][h], sm_m[1][h]), fmaxf(sm_m[2][h], sm_m[3][h]));
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
    split_tail<T, D>(ta, u);
}

template <typename T, int D, int G>
static hipError_t launch_one(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    const SplitTailArgs<T> ta = make_tail_args<T>(p, io, n, n_caches);
    const SplitGroup gr = make_split_group(p, table, p.units * ta.c_active);
    const float scale_log2 = 1.4426950408889634f / sqrtf((float)D);
    hipLaunchKernelGGL((split_valu_kernel<T, D, G>), dim3(p.units * ta.c_active * n_caches), dim3(256), 0, s, ta,
                       scale_log2, gr);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && !ta.fused_tail && ta.c_active > 1) e = launch_split_finish<T, D>(ta, p.units, gr, n_caches, s);
    return e;
}

template <typename T, int D>
static hipError_t launch_g(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    switch (p.G) {
    case 1: return launch_one<T, D, 1>(p, io, n, s, table, n_caches);
    case 2: return launch_one<T, D, 2>(p, io, n, s, table, n_caches);
    case 3: return launch_one<T, D, 3>(p, io, n, s, table, n_caches);
    case 4: return launch_one<T, D, 4>(p, io, n, s, table, n_caches);
    case 5: return launch_one<T, D, 5>(p, io, n, s, table, n_caches);
    case 6: return launch_one<T, D, 6>(p, io, n, s, table, n_caches);
    case 7: return launch_one<T, D, 7>(p, io, n, s, table, n_caches);
    case 8: return launch_one<T, D, 8>(p, io, n, s, table, n_caches);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_split_valu(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table, int n_caches)
{
    if (p.dtype == 0)
        return p.D == 64 ? launch_g<float, 64>(p, io, n, s, table, n_caches) : launch_g<float, 128>(p, io, n, s, table, n_caches);
    return p.D == 64 ? launch_g<bf16_t, 64>(p, io, n, s, table, n_caches) : launch_g<bf16_t, 128>(p, io, n, s, table, n_caches);
}

size_t split_table_entry_bytes() { return sizeof(SplitTailArgs<float>); }

void split_table_entry(const Plan &p, void *dst)
{
    static_assert(sizeof(SplitTailArgs<float>) == sizeof(SplitTailArgs<bf16_t>), "one table layout for both element types");
    static_assert(sizeof(SplitTailArgs<float>) <= kTableEntryMax && sizeof(SplitTailArgs<float>) % 4 == 0, "entry travels as a kernel argument");
    const StepIo none = {nullptr, nullptr, nullptr, nullptr, nullptr};
    if (p.dtype == 0) {
        SplitTailArgs<float> a = make_tail_args<float>(p, none, p.N);
        a.lu = p.lu; // a mask may come into force after the table was written
        memcpy(dst, &a, sizeof(a));
    } else {
        SplitTailArgs<bf16_t> a = make_tail_args<bf16_t>(p, none, p.N);
        a.lu = p.lu;
        memcpy(dst, &a, sizeof(a));
    }
}

} // namespace lf
