// Matrix-core streaming core shared by the split-K kernel and the unit-resident fused
// kernel (bf16, head_dim 128, wave64, gfx950).
//
// A wave streams 16-slot tiles of K and V exactly once with 128-bit loads that land
// directly in MFMA operand layouts (no LDS staging, no transposes through memory).
// Every load instruction of a wave covers whole 128-byte lines (8 K rows x one line, or
// 4 V rows x two lines): the per-CU limit on outstanding line requests, not HBM, is what
// caps a compute unit's streaming rate, and half-line requests would waste a third of it.
//
//   S^T = K Q^T      8 x v_mfma_f32_16x16x32_bf16 (two half-used products per 8 slots, see
//                    below), rows = slots, cols = 16 (padded) heads
//   p   = 2^(t - m)  online softmax per head in fp32, reference m raised lazily  (eq. 1)
//   O  += P V        8 x v_mfma_f32_16x16x16_bf16, P as bf16 hi (+ lo) parts
//   code             8-bit log2 code of ||v_i||_1 * p_h,i for the eviction screening (eq. 6);
//                    log2 ||v_i||_1 comes from a small side array kept current on insert
//
// Lane naming: g = lane >> 4 (0..3), r = lane & 15.
//
// K operand.  For the lanes covering one K row to form a full line, lane (g, r) reads row
// rho = r >> 1 of an 8-row group, 16-byte chunk 2g + b (b = r & 1) of line L.  As an MFMA A
// operand that makes "row" r = (rho, b) and contraction index k = 8g + j stand for channel
// 64L + 8(2g + b) + j, which depends on b.  Two products per group, one with the Q chunks
// of b = 0 and one with those of b = 1, each produce the right half-dot-product in the rows
// of their own b; the halves of a slot sit in adjacent accumulator registers of one lane,
// so a single add per slot finishes the logit.  The spare products are free: the matrix
// pipe idles most of the time in this HBM-bound kernel.
//
// Within a tile a lane (g, head) ends up with the logits of slot offsets
//   s(e) = 8 (e >> 1) + 2 g + (e & 1),  e = 0..3,
// and everything per-slot that the kernels keep (codes, stash, log2 norms) is stored in
// "position" order p = 4 g + e inside each 16-slot tile.
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
// The running softmax reference is raised only when a logit exceeds it by more than this
// (log2 units): p stays below 2^kMaxSlack, far inside fp32/bf16 range, and the common
// path needs no cross-lane traffic at all.
constexpr float kMaxSlack = 8.f;
// Reference of a softmax state that has seen no valid slot yet: finite, so that a tile of
// masked slots only (logits -inf) gives p = 2^(-inf - kNoRef) = 0 rather than NaN, and so
// far below any logit that the first valid one replaces it (weights 2^(kNoRef - m) = 0).
constexpr float kNoRef = -3.0e38f;

// position of a slot inside its 16-slot tile, and back
__host__ __device__ __forceinline__ int pos_of_slot(int s) { return 4 * ((s >> 1) & 3) + 2 * ((s >> 3) & 1) + (s & 1); }
__host__ __device__ __forceinline__ int slot_of_pos(int p) { return 8 * ((p >> 1) & 1) + 2 * (p >> 2) + (p & 1); }

// Pointers of the streaming core live in the global address space by type: a pointer that
// reached the kernel through device memory (the table of a grouped launch) is generic to the
// compiler, generic accesses become FLAT instructions, and a FLAT load can only be waited for
// together with every other outstanding one -- which would undo the rotation of register
// tiles below.
typedef __attribute__((address_space(1))) const uint16_t *g_cu16p;
typedef __attribute__((address_space(1))) const float *g_cf32p;
typedef __attribute__((address_space(1))) uint16_t *g_u16p;
typedef __attribute__((address_space(1))) float *g_f32p;
typedef __attribute__((address_space(1))) const u32x4 *g_cu32x4p;
typedef __attribute__((address_space(1))) const f32x4 *g_cf32x4p;
typedef __attribute__((address_space(1))) u32x2 *g_u32x2p;
typedef __attribute__((address_space(1))) const u32x2 *g_cu32x2p;
typedef __attribute__((address_space(1))) uint32_t *g_u32p;

struct TileRegs {
    u32x4 k[2][2]; // k[a][L]: row 8a + (r >> 1), line L, chunk 2g + (r & 1)
    u32x4 v[4];    // v[e]: row s(e), channels 8r .. 8r + 7
    f32x4 lu;      // log2 ||v||_1 of the lane's four slots (positions 4g .. 4g + 3)
};

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2 f = {lo, hi};
    bf16x2 b = __builtin_convertvector(f, bf16x2);
    return __builtin_bit_cast(uint32_t, b);
}

// KNAT: K in the natural A-operand layout -- lane (g, r) reads row r of the tile, channels
//       32c + 8g .. +7 for c = 0..3 (16 rows x 64 B per instruction: half lines), one product of
//       four MFMAs gives the whole logit, and a lane's four slots are 4g .. 4g + 3.  Half the
//       matrix instructions of the full-line scheme and no joining adds, at the price of the
//       half-line loads: right for the multi-query kernel, which is bound by arithmetic and not
//       by a compute unit's request rate.  (No per-slot side data exists in that layout.)
// MASKED: an explicit validity mask may be in force (NaN entries of the side array)
// CAUSAL: every column (lane r) has its own row limit: it sees slots below `limit` only
// MAXFREE: the softmax of Alg. 1 as printed (Sec. 3.4, modification 2): no running reference,
//          p = 2^t in fp32; overflows once a logit passes 2^128.  For A/B measurement.
template <int NWAVES, bool HILO, int STASH, bool MASKED = false, bool CAUSAL = false, bool MAXFREE = false, bool KNAT = false>
struct MfmaStreamer {
    static_assert(!KNAT || STASH == kStashNone, "the natural K layout keeps no per-slot side data");
    static constexpr int D = 128;
    // per-wave state
    u32x4 qreg[2][2]; // qreg[L][b]: head r, channels 64L + 8(2g + b) .. +7
    f32x4 oacc[8];    // oacc[dd][v]: head 4g + v, channel 8r + dd
    float m, l;       // reference (log2 domain) and lane-partial denominator of head r
    // geometry
    g_cu16p Ku, Vu;
    g_cf32p lu_unit;      // [ntiles * 16] log2 ||v||_1 in position order
    int start, end, G, g, r;
    int limit; // CAUSAL: first slot column r does not see
    float scale_log2;
    // stash sinks
    g_u16p gs_w;      // kStashGlobal: [tile][G][16 positions] bf16
    g_f32p gs_m;      // kStashGlobal: [tile][G]
    uint8_t *ls_code; // kStashLds: [G][code_stride] bytes, position order, counted from `start`
    float *ls_ref;    // kStashLds: [tile][G], tiles counted from `start`
    int code_stride;

    __device__ __forceinline__ void init(g_cu16p q_unit, int G_, int lane, float scale)
    {
        G = G_; g = lane >> 4; r = lane & 15; scale_log2 = scale;
#pragma unroll
        for (int L = 0; L < 2; ++L)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                qreg[L][b] = u32x4{0u, 0u, 0u, 0u};
                if (r < G) qreg[L][b] = *(g_cu32x4p)(q_unit + (size_t)r * D + 64 * L + 8 * (2 * g + b));
            }
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) oacc[dd] = f32x4{0.f, 0.f, 0.f, 0.f};
        m = MAXFREE ? 0.f : kNoRef;
        l = 0.f;
    }

    // One column of a multi-query product: the query row at q_col (nullptr = unused column),
    // which sees slots [0, limit_) only.
    __device__ __forceinline__ void init_column(g_cu16p q_col, int limit_, int lane, float scale)
    {
        G = 16; g = lane >> 4; r = lane & 15; scale_log2 = scale; limit = q_col ? limit_ : 0;
#pragma unroll
        for (int L = 0; L < 2; ++L)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                qreg[L][b] = u32x4{0u, 0u, 0u, 0u};
                // KNAT: qreg[c >> 1][c & 1] holds channels 32c + 8g .. +7
                if (q_col) qreg[L][b] = *(g_cu32x4p)(q_col + (KNAT ? 32 * (2 * L + b) + 8 * g : 64 * L + 8 * (2 * g + b)));
            }
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) oacc[dd] = f32x4{0.f, 0.f, 0.f, 0.f};
        m = MAXFREE ? 0.f : kNoRef;
        l = 0.f;
    }

    __device__ __forceinline__ int slot_off(int e) const { return KNAT ? 4 * g + e : 8 * (e >> 1) + 2 * g + (e & 1); }

    // K/V are read once and never again by a decode step: non-temporal.  The multi-query
    // (CAUSAL) kernel has several waves walk the same rows: ordinary loads, so that the caches
    // keep the lines for the other waves.
    static __device__ __forceinline__ u32x4 stream_load(g_cu32x4p p)
    {
        return CAUSAL ? *p : __builtin_nontemporal_load(p);
    }

    // RAGGED clamps rows to the valid prefix (a full tile needs no clamp)
    template <bool RAGGED> __device__ __forceinline__ void load_tile(TileRegs &t, int ti) const
    {
        const int base = start + ti * kTile;
        const int last = end - 1;
        // side array first: loads return in order, and its first use (the mask test right
        // after the logits) must not have to wait for this tile's V rows
        if (STASH != kStashNone) t.lu = *(g_cf32x4p)(lu_unit + base + 4 * g);
        if (KNAT) {
            int krow = base + r;
            if (RAGGED) krow = min(krow, last);
#pragma unroll
            for (int c = 0; c < 4; ++c) t.k[c >> 1][c & 1] = stream_load((g_cu32x4p)(Ku + (size_t)krow * D + 32 * c + 8 * g));
        } else {
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                int krow = base + 8 * a + (r >> 1);
                if (RAGGED) krow = min(krow, last);
#pragma unroll
                for (int L = 0; L < 2; ++L)
                    t.k[a][L] = stream_load((g_cu32x4p)(Ku + (size_t)krow * D + 64 * L + 8 * (2 * g + (r & 1))));
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int vrow = base + slot_off(e);
            if (RAGGED) vrow = min(vrow, last);
            t.v[e] = stream_load((g_cu32x4p)(Vu + (size_t)vrow * D + 8 * r));
        }
    }

    // B operand of P V product dd (channel 8r + dd): v_perm picks, from a lane's four V rows, the bf16 pairs of
    // positions (4g, 4g + 1) and (4g + 2, 4g + 3)
    static __device__ __forceinline__ s16x4 v_operand(const TileRegs &t, int dd)
    {
        const uint32_t sel = (dd & 1) ? 0x07060302u : 0x05040100u;
        const int w = dd >> 1;
        const uint32_t v01 = __builtin_amdgcn_perm(t.v[1][w], t.v[0][w], sel);
        const uint32_t v23 = __builtin_amdgcn_perm(t.v[3][w], t.v[2][w], sel);
        return __builtin_bit_cast(s16x4, u32x2{v01, v23});
    }
    // The eight operands built once, in place of the V rows they come from (same number of registers):
    // afterwards t.v[i] holds the operands of products 2i and 2i + 1.  For kernels that take several
    // products through one tile (compute_core<.., .., VPRE = true>).
    static __device__ __forceinline__ void build_v_in_place(TileRegs &t)
    {
        u32x2 vb[8];
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) vb[dd] = __builtin_bit_cast(u32x2, v_operand(t, dd));
#pragma unroll
        for (int i = 0; i < 4; ++i) t.v[i] = u32x4{vb[2 * i].x, vb[2 * i].y, vb[2 * i + 1].x, vb[2 * i + 1].y};
    }

    // RAGGED: the tile may reach past `end`; rows loaded from the clamped address are zeroed
    template <bool RAGGED> __device__ __forceinline__ void zero_ragged(TileRegs &t, int ti) const
    {
        const int base = start + ti * kTile;
        if (RAGGED) {
            if (KNAT) {
                if (base + r >= end) t.k[0][0] = t.k[0][1] = t.k[1][0] = t.k[1][1] = u32x4{0u, 0u, 0u, 0u};
            } else {
#pragma unroll
                for (int a = 0; a < 2; ++a)
                    if (base + 8 * a + (r >> 1) >= end) t.k[a][0] = t.k[a][1] = u32x4{0u, 0u, 0u, 0u};
            }
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + slot_off(e) >= end) t.v[e] = u32x4{0u, 0u, 0u, 0u};
        }
    }

    template <bool RAGGED> __device__ __forceinline__ void compute_tile(TileRegs &t, int ti)
    {
        zero_ragged<RAGGED>(t, ti);
        compute_core<RAGGED, CAUSAL, false>(t, ti);
    }

    // The two halves of a tile (logits, then everything else), callable apart so that a kernel with several products per wave can have
    // the logits of all of them on the matrix pipe before the vector work of the first begins.
    __device__ __forceinline__ void logits(const TileRegs &t, float (&s)[4]) const
    {
        // ---- S^T = K Q^T: per 8-row group, one product per chunk parity b
        if (KNAT) {
            f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int c = 0; c < 4; ++c)
                d = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, t.k[c >> 1][c & 1]),
                                                            __builtin_bit_cast(bf16x8, qreg[c >> 1][c & 1]), d, 0, 0, 0);
            // accumulator rows 4g + v are slots 4g + v
            s[0] = d[0]; s[1] = d[1]; s[2] = d[2]; s[3] = d[3];
        }
#pragma unroll
        for (int a = 0; a < (KNAT ? 0 : 2); ++a) {
            f32x4 d0 = {0.f, 0.f, 0.f, 0.f}, d1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int L = 0; L < 2; ++L) {
                const bf16x8 ka = __builtin_bit_cast(bf16x8, t.k[a][L]);
                d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, __builtin_bit_cast(bf16x8, qreg[L][0]), d0, 0, 0, 0);
                d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, __builtin_bit_cast(bf16x8, qreg[L][1]), d1, 0, 0, 0);
            }
            // accumulator rows 4g + v = (rho = 2g + (v >> 1), b = v & 1)
            s[2 * a + 0] = d0[0] + d1[1];
            s[2 * a + 1] = d0[2] + d1[3];
        }
    }

    // Two tiles per P V product (multi-query kernels; single bf16 weights, t.v built in place).  The weights of
    // a tile are left in fp32 so that the second tile of a pair can still move the reference: it rescales the
    // first tile's pending weights along with the sums.  Then ONE matrix instruction per 16 channels contracts
    // over the 32 slots of both tiles (v_mfma_f32_16x16x32_bf16: lane (g, r) supplies k = 8g .. 8g+7, taken
    // here as slots 4g .. 4g+3 of the first tile followed by the same slots of the second, for both operands)
    // where the one-tile form needs two half-rate 16x16x16 instructions.
    __device__ __forceinline__ void tile_weights(int ti, float (&s)[4], bool cmask_now, float (&p)[4], float *p_prev)
    {
        const int base = start + ti * kTile;
        if (cmask_now) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + slot_off(e) >= limit) s[e] = -INFINITY;
        }
        const float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])) * scale_log2;
        if (!MAXFREE && __any(mx > m + kMaxSlack)) {
            float mw = fmaxf(mx, __shfl_xor(mx, 16));
            mw = fmaxf(mw, __shfl_xor(mw, 32));
            const float m_new = (mw > m + kMaxSlack) ? mw : m;
            const float a = fast_exp2(m - m_new);
            l *= a;
            if (p_prev) { // weights of the pair's first tile, this lane's own column
#pragma unroll
                for (int e = 0; e < 4; ++e) p_prev[e] *= a;
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float av = __shfl(a, 4 * g + v);
#pragma unroll
                for (int dd = 0; dd < 8; ++dd) oacc[dd][v] *= av;
            }
            m = m_new;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            p[e] = fast_exp2(fmaf(s[e], scale_log2, -m));
            l += p[e];
        }
    }
    __device__ __forceinline__ void pv_pair(const TileRegs &t0, const TileRegs &t1, const float (&p0)[4], const float (&p1)[4])
    {
        const u32x4 pa = {pack_bf16x2(p0[0], p0[1]), pack_bf16x2(p0[2], p0[3]), pack_bf16x2(p1[0], p1[1]), pack_bf16x2(p1[2], p1[3])};
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            const int i = dd >> 1, j = 2 * (dd & 1);
            const u32x4 vb = {t0.v[i][j], t0.v[i][j + 1], t1.v[i][j], t1.v[i][j + 1]};
            oacc[dd] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, pa), __builtin_bit_cast(bf16x8, vb), oacc[dd], 0, 0, 0);
        }
    }

    // One tile of one product, from rows already cleaned (zero_ragged).
    // CMASK: the column's causal row limit may apply; `cmask_now` (uniform over the wave) says whether this tile
    //        needs the test at all -- tiles that every column of the wave sees whole skip it
    // VPRE:  t.v already holds the P V operands (build_v_in_place)
    template <bool RAGGED, bool CMASK, bool VPRE> __device__ __forceinline__ void compute_core(const TileRegs &t, int ti, bool cmask_now = true)
    {
        float s[4];
        logits(t, s);
        finish_tile<RAGGED, CMASK, VPRE>(t, ti, s, cmask_now);
    }

    template <bool RAGGED, bool CMASK, bool VPRE>
    __device__ __forceinline__ void finish_tile(const TileRegs &t, int ti, float (&s)[4], bool cmask_now = true)
    {
        const int base = start + ti * kTile;
        if (RAGGED) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + slot_off(e) >= end) s[e] = -INFINITY;
        }
        if (CMASK && cmask_now) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (base + slot_off(e) >= limit) s[e] = -INFINITY;
        }
        // ---- explicit mask (Alg. 1's M): a slot whose side-array entry is NaN is invalid;
        // its logit becomes -inf, hence p = 0 (its V row is kept finite by the mask setter)
        if (MASKED && STASH != kStashNone) {
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] = (t.lu[e] != t.lu[e]) ? -INFINITY : s[e];
        }
        // ---- online softmax with a lazily raised reference
        const float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3])) * scale_log2;
        if (!MAXFREE && __any(mx > m + kMaxSlack)) { // rare: first tile, or a logit far above everything so far
            float mw = fmaxf(mx, __shfl_xor(mx, 16));
            mw = fmaxf(mw, __shfl_xor(mw, 32));
            const float m_new = (mw > m + kMaxSlack) ? mw : m;
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
        for (int e = 0; e < 4; ++e) {
            lg[e] = fmaf(s[e], scale_log2, -m); // log2 of p; -inf for masked slots
            p[e] = fast_exp2(lg[e]);
            l += p[e];
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
        // ---- O += P V, channel 8r + dd per product; contraction index 4g + e = position
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            const s16x4 vb = VPRE ? __builtin_bit_cast(s16x4, u32x2{t.v[dd >> 1][2 * (dd & 1)], t.v[dd >> 1][2 * (dd & 1) + 1]})
                                  : v_operand(t, dd);
            oacc[dd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_hi, vb, oacc[dd], 0, 0, 0);
            if (HILO) oacc[dd] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(p_lo, vb, oacc[dd], 0, 0, 0);
        }
        if (STASH == kStashGlobal) {
            if (r < G) {
                float w[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) w[e] = fast_exp2(t.lu[e] + lg[e]); // ||v||_1 * p
                const size_t rec = (size_t)(base / kTile) * G + r;
                *(g_u32x2p)(gs_w + rec * kTile + 4 * g) = u32x2{pack_bf16x2(w[0], w[1]), pack_bf16x2(w[2], w[3])};
                if (g == 0) gs_m[rec] = m;
            }
        }
        if (STASH == kStashLds) {
            uint32_t code = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                // 4 * (bias - log2(u p)), rounded, clamped to a byte
                float c = __builtin_amdgcn_fmed3f(rintf(fmaf(t.lu[e] + lg[e], -4.f, 4.f * kCodeBias)), 0.f, 255.f);
                // a position past the last slot carries the clamp code whatever its side-array entry holds:
                // the screening sends clamped codes through its exact path, which knows the slot count
                if (RAGGED && base + slot_off(e) >= end) c = 255.f;
                code = __builtin_amdgcn_cvt_pk_u8_f32(c, e, code);
            }
            if (r < G) {
                *(uint32_t *)(ls_code + (size_t)r * code_stride + (base - start) + 4 * g) = code;
                if (g == 0) ls_ref[((base - start) / kTile) * G + r] = m;
            }
        }
    }

    // Stream this wave's share of [start, end): wave w owns tiles w, w + NWAVES, ...
    // (A static split keeps every sum in a fixed order: results are bit-reproducible.
    // Handing tiles out dynamically was tried -- the older wave of a SIMD finishes ~40 %
    // ahead of the younger one -- and bought nothing: the compute unit's request rate, not
    // the number of waves still streaming, sets the pace.  Starting every workgroup at a
    // different, hashed position of its tile list was tried as well, against memory-channel
    // hot spots: it is 12-15 % slower (173 -> 195 us at 256 units x 8192 slots).  Workgroups
    // that walk their units in step, at equal offsets of 2 MiB-strided units, are the
    // pattern the channel hashing spreads best.)
    // Three register tiles rotate: while one is consumed the other two are in flight; the
    // steady-state body has no branch between a load and its use, so each wait covers
    // exactly the oldest tile.
    // The first three tiles of a wave's share can be requested ahead of run() (a kernel that has other
    // latencies to sit out before streaming, such as finding out which slot to insert into): returns
    // whether it did (only shares of at least three full tiles are started this way).  The caller
    // re-requests a tile whose rows it changes afterwards.
    __device__ __forceinline__ bool request_first_tiles(int wave, TileRegs &ta, TileRegs &tb, TileRegs &tc) const
    {
        const int nfull = (end - start) / kTile;
        const int n_my = (nfull > wave) ? (nfull - wave + NWAVES - 1) / NWAVES : 0;
        if (n_my < 3) return false;
        load_tile<false>(ta, wave);
        load_tile<false>(tb, wave + NWAVES);
        load_tile<false>(tc, wave + NWAVES * 2);
        return true;
    }

    __device__ __forceinline__ void run(int wave)
    {
        TileRegs ta, tb, tc;
        run(wave, ta, tb, tc, false);
    }

    // requested: ta, tb, tc already hold (requests for) the wave's first three tiles
    __device__ __forceinline__ void run(int wave, TileRegs &ta, TileRegs &tb, TileRegs &tc, bool requested)
    {
        const int nfull = (end - start) / kTile;
        const bool ragged = (end - start) % kTile != 0;
        const int n_my = (nfull > wave) ? (nfull - wave + NWAVES - 1) / NWAVES : 0;
        if (n_my >= 3) {
            // prologue loads are unconditional inside this branch: the waits in the loop
            // then cover exactly the oldest tile and leave the younger loads in flight
            if (!requested) {
                load_tile<false>(ta, wave);
                load_tile<false>(tb, wave + NWAVES);
                load_tile<false>(tc, wave + NWAVES * 2);
            }
            int i = 0;
            for (; i + 5 < n_my; i += 3) {
                compute_tile<false>(ta, wave + NWAVES * i);
                load_tile<false>(ta, wave + NWAVES * (i + 3));
                compute_tile<false>(tb, wave + NWAVES * (i + 1));
                load_tile<false>(tb, wave + NWAVES * (i + 4));
                compute_tile<false>(tc, wave + NWAVES * (i + 2));
                load_tile<false>(tc, wave + NWAVES * (i + 5));
            }
            // 3 to 5 tiles remain; the first three are already on their way
            compute_tile<false>(ta, wave + NWAVES * i);
            if (i + 3 < n_my) load_tile<false>(ta, wave + NWAVES * (i + 3));
            compute_tile<false>(tb, wave + NWAVES * (i + 1));
            if (i + 4 < n_my) load_tile<false>(tb, wave + NWAVES * (i + 4));
            compute_tile<false>(tc, wave + NWAVES * (i + 2));
            if (i + 3 < n_my) compute_tile<false>(ta, wave + NWAVES * (i + 3));
            if (i + 4 < n_my) compute_tile<false>(tb, wave + NWAVES * (i + 4));
        } else {
            // one or two tiles (short spans: small caches split over many workgroups), plus
            // possibly the ragged one: every load is issued before the first tile is consumed,
            // one trip to memory instead of one per tile
            const bool mine = ragged && wave == nfull % NWAVES;
            if (n_my >= 1) load_tile<false>(ta, wave);
            if (n_my >= 2) load_tile<false>(tb, wave + NWAVES);
            if (mine) load_tile<true>(tc, nfull);
            if (n_my >= 1) compute_tile<false>(ta, wave);
            if (n_my >= 2) compute_tile<false>(tb, wave + NWAVES);
            if (mine) compute_tile<true>(tc, nfull);
            return;
        }
        if (ragged && wave == nfull % NWAVES) {
            load_tile<true>(ta, nfull);
            compute_tile<true>(ta, nfull);
        }
    }
};

} // namespace lf
