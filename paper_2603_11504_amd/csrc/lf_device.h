// Device-side helpers shared by the LongFlow kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lf {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

struct bf16_t { uint16_t bits; };   // storage-only bfloat16

__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// float -> bfloat16 bits, round to nearest even (NaN kept quiet)
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float x)
{
    uint32_t u = __float_as_uint(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// weight of a partial state whose reference is `m` when merged under reference `M`;
// an empty state carries m = -inf and weighs nothing
__device__ __forceinline__ float merge_weight(float m, float M)
{
    return (m == -INFINITY) ? 0.f : fast_exp2(m - M);
}

// ---- DPP rotations inside a row of 16 lanes: all-reduce without LDS traffic
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_f32<0x128>(x); // row_ror:8
    x += dpp_f32<0x124>(x); // row_ror:4
    x += dpp_f32<0x122>(x); // row_ror:2
    x += dpp_f32<0x121>(x); // row_ror:1
    return x;
}
__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, dpp_f32<0x128>(x));
    x = fmaxf(x, dpp_f32<0x124>(x));
    x = fmaxf(x, dpp_f32<0x122>(x));
    x = fmaxf(x, dpp_f32<0x121>(x));
    return x;
}

// ---- element loads: EPL consecutive elements of a row into floats
template <typename T, int EPL> struct RowChunk;

template <> struct RowChunk<float, 4> {
    float v[4];
    __device__ __forceinline__ void load(const float *p) { f32x4 t = *(const f32x4 *)p; v[0]=t.x; v[1]=t.y; v[2]=t.z; v[3]=t.w; }
    __device__ __forceinline__ void zero() { for (int i = 0; i < 4; ++i) v[i] = 0.f; }
};
template <> struct RowChunk<float, 8> {
    float v[8];
    __device__ __forceinline__ void load(const float *p) {
        f32x4 a = *(const f32x4 *)p, b = *(const f32x4 *)(p + 4);
        v[0]=a.x; v[1]=a.y; v[2]=a.z; v[3]=a.w; v[4]=b.x; v[5]=b.y; v[6]=b.z; v[7]=b.w; }
    __device__ __forceinline__ void zero() { for (int i = 0; i < 8; ++i) v[i] = 0.f; }
};
template <> struct RowChunk<bf16_t, 4> {
    float v[4];
    __device__ __forceinline__ void load(const bf16_t *p) {
        u32x2 t = *(const u32x2 *)p;
        v[0]=bf16_lo(t.x); v[1]=bf16_hi(t.x); v[2]=bf16_lo(t.y); v[3]=bf16_hi(t.y); }
    __device__ __forceinline__ void zero() { for (int i = 0; i < 4; ++i) v[i] = 0.f; }
};
template <> struct RowChunk<bf16_t, 8> {
    float v[8];
    __device__ __forceinline__ void load(const bf16_t *p) {
        u32x4 t = *(const u32x4 *)p;
        v[0]=bf16_lo(t.x); v[1]=bf16_hi(t.x); v[2]=bf16_lo(t.y); v[3]=bf16_hi(t.y);
        v[4]=bf16_lo(t.z); v[5]=bf16_hi(t.z); v[6]=bf16_lo(t.w); v[7]=bf16_hi(t.w); }
    __device__ __forceinline__ void zero() { for (int i = 0; i < 8; ++i) v[i] = 0.f; }
};

__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16_t x) { return __uint_as_float((uint32_t)x.bits << 16); }
__device__ __forceinline__ void store_elem(float *p, float x) { *p = x; }
__device__ __forceinline__ void store_elem(bf16_t *p, float x) { p->bits = (uint16_t)f32_to_bf16_bits(x); }

} // namespace lf
