// Kernels off the per-step path: value-norm side array at cache init, on-demand score
// read-back, small fills.
#include <cstring>
#include <mutex>

#include "lf_device.h"
#include "lf_host.h"
#include "lf_split_tail.h"

namespace lf {

// log2 ||v||_1 of rows [0, n_rows) of every unit (prefill), one 16-lane row per cache row
__global__ __launch_bounds__(256) void l1norm_kernel(const uint16_t *__restrict__ Vc, float *__restrict__ lu,
                                                      int units, int N, int n_rows, int lu_stride)
{
    const int lane16 = threadIdx.x & 15;
    const long long total = (long long)units * n_rows;
    for (long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4); row < total; row += (long long)gridDim.x * 16) {
        const int u = (int)(row / n_rows), slot = (int)(row % n_rows);
        const u32x4 vv = *(const u32x4 *)(Vc + ((size_t)u * N + slot) * 128 + 8 * lane16);
        float a1 = fabsf(bf16_lo(vv.x)) + fabsf(bf16_hi(vv.x)) + fabsf(bf16_lo(vv.y)) + fabsf(bf16_hi(vv.y)) +
                   fabsf(bf16_lo(vv.z)) + fabsf(bf16_hi(vv.z)) + fabsf(bf16_lo(vv.w)) + fabsf(bf16_hi(vv.w));
        a1 = row16_sum(a1);
        if (lane16 == 0) lu[(size_t)u * lu_stride + (slot & ~15) + tail_pos_of_slot(slot & 15)] = __builtin_amdgcn_logf(a1);
    }
}
hipError_t launch_l1norms(const Plan &p, int n_rows, hipStream_t s)
{
    const long long total = (long long)p.units * n_rows;
    long long blocks = (total + 15) / 16;
    if (blocks > 65536) blocks = 65536;
    if (blocks < 1) return hipSuccess;
    hipLaunchKernelGGL(l1norm_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const uint16_t *)p.v_cache, p.lu,
                       p.units, p.N, n_rows, p.ntiles * kTile);
    return hipGetLastError();
}

__global__ void fill_i32_kernel(int32_t *dst, int count, int32_t value)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) dst[i] = value;
}
hipError_t launch_fill_i32(int32_t *dst, int count, int32_t value, hipStream_t s)
{
    hipLaunchKernelGGL(fill_i32_kernel, dim3((count + 255) / 256), dim3(256), 0, s, dst, count, value);
    return hipGetLastError();
}

struct TableEntryBlob { uint32_t w[kTableEntryMax / 4]; };
__global__ void table_entry_kernel(uint32_t *dst, const TableEntryBlob e, int words)
{
    const int i = threadIdx.x;
    if (i < words) dst[i] = e.w[i];
}
hipError_t launch_table_entry(void *dst, const void *entry, size_t bytes, hipStream_t s)
{
    if (bytes > kTableEntryMax || (bytes & 3u)) return hipErrorInvalidValue;
    TableEntryBlob e;
    memset(&e, 0, sizeof(e));
    memcpy(&e, entry, bytes);
    hipLaunchKernelGGL(table_entry_kernel, dim3(1), dim3(kTableEntryMax / 4), 0, s, (uint32_t *)dst, e, (int)(bytes / 4));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Explicit validity mask (the vector M of Alg. 1), off the per-step path.  One 16-lane row
// per cache row: an invalid slot gets NaN in the side array and zeroed K/V rows (a zero
// weight times a non-finite value would still poison the P V product), a valid one gets
// log2 ||v||_1.  The lowest invalid slot of each unit becomes its pending slot.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void mask_kernel(T *__restrict__ Kc, T *__restrict__ Vc,
                                                    const uint8_t *__restrict__ mask, float *__restrict__ lu,
                                                    int32_t *__restrict__ first_hole, int units, int N, int lu_stride)
{
    constexpr int EPL = D / 16;
    const int lane16 = threadIdx.x & 15;
    const long long total = (long long)units * N;
    for (long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4); row < total; row += (long long)gridDim.x * 16) {
        const int u = (int)(row / N), slot = (int)(row % N);
        T *kr = Kc + (size_t)row * D + lane16 * EPL;
        T *vr = Vc + (size_t)row * D + lane16 * EPL;
        float val;
        if (mask[row]) {
            float a1 = 0.f;
#pragma unroll
            for (int e = 0; e < EPL; ++e) a1 += fabsf(to_f32(vr[e]));
            val = __builtin_amdgcn_logf(row16_sum(a1));
        } else {
#pragma unroll
            for (int e = 0; e < EPL; ++e) { store_elem(kr + e, 0.f); store_elem(vr + e, 0.f); }
            val = __builtin_nanf("");
            if (lane16 == 0) atomicMin(&first_hole[u], slot);
        }
        if (lane16 == 0) lu[(size_t)u * lu_stride + (slot & ~15) + tail_pos_of_slot(slot & 15)] = val;
    }
}

__global__ void mask_pending_kernel(const int32_t *first_hole, int32_t *pending, int units, int N)
{
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u < units && first_hole[u] < N) pending[u] = first_hole[u];
}

// validity of every slot as bytes: the prefix [0, n) without an explicit mask, else the
// non-NaN entries of the side array
__global__ void get_mask_kernel(const float *__restrict__ lu, uint8_t *__restrict__ mask, int units, int N, int n,
                                int lu_stride, int masked)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)units * N) return;
    const int u = (int)(i / N), slot = (int)(i % N);
    bool valid = slot < n;
    if (valid && masked) {
        const float x = lu[(size_t)u * lu_stride + (slot & ~15) + tail_pos_of_slot(slot & 15)];
        valid = x == x;
    }
    mask[i] = valid ? 1 : 0;
}

hipError_t launch_get_mask(const Plan &p, int n, uint8_t *mask, hipStream_t s)
{
    const long long total = (long long)p.units * p.N;
    hipLaunchKernelGGL(get_mask_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p.lu, mask, p.units,
                       p.N, n, p.ntiles * kTile, p.masked ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_set_mask(const Plan &p, const uint8_t *mask, hipStream_t s)
{
    hipError_t e = launch_fill_i32(p.first_hole, p.units, 0x7fffffff, s);
    if (e != hipSuccess) return e;
    const long long total = (long long)p.units * p.N;
    long long blocks = (total + 15) / 16;
    if (blocks > 65536) blocks = 65536;
#define LF_MK(T, DD)                                                                              \
    hipLaunchKernelGGL((mask_kernel<T, DD>), dim3((unsigned)blocks), dim3(256), 0, s, (T *)p.k_cache, \
                       (T *)p.v_cache, mask, p.lu, p.first_hole, p.units, p.N, p.ntiles * kTile)
    if (p.dtype == 0) { if (p.D == 64) LF_MK(float, 64); else LF_MK(float, 128); }
    else              { if (p.D == 64) LF_MK(bf16_t, 64); else LF_MK(bf16_t, 128); }
#undef LF_MK
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(mask_pending_kernel, dim3((p.units + 255) / 256), dim3(256), 0, s, p.first_hole, p.pending,
                       p.units, p.N);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Score read-back (S_final_loss of Alg. 1), off the per-step path: one wave per slot,
// double-precision arithmetic; fp32 result with 0 for invalid slots (longflow_scores), or
// the double itself with +inf for invalid slots (input of the batch eviction below).
// ---------------------------------------------------------------------------------------
template <typename T, int D, typename OUT>
__global__ __launch_bounds__(256) void scores_kernel(const T *__restrict__ Kc, const T *__restrict__ Vc,
                                                      const T *__restrict__ q_last, int n, int N, int G,
                                                      const float *__restrict__ fin_m,
                                                      const float *__restrict__ fin_l,
                                                      OUT *__restrict__ scores, int chunks,
                                                      const float *__restrict__ lu_mask, int lu_stride)
{
    __shared__ float sM[kMaxGroup], sL[kMaxGroup];
    const int u = blockIdx.x / chunks, ch = blockIdx.x % chunks;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < G) { sM[tid] = fin_m[(size_t)u * G + tid]; sL[tid] = fin_l[(size_t)u * G + tid]; }
    __syncthreads();
    const int per = (N + chunks - 1) / chunks;
    const int lo = ch * per, hi = min(lo + per, N);
    for (int slot = lo + wave; slot < hi; slot += 4) {
        OUT r = sizeof(OUT) == 8 ? (OUT)INFINITY : (OUT)0;
        // lu_mask: explicit mask in force, NaN marks an invalid slot (score 0, as in Alg. 1)
        bool valid = slot < n;
        if (valid && lu_mask) {
            const float x = lu_mask[(size_t)u * lu_stride + (slot & ~15) + tail_pos_of_slot(slot & 15)];
            valid = x == x;
        }
        if (valid) {
            const double v = tail_exact_score<T, D>(Kc + ((size_t)u * N + slot) * D, Vc + ((size_t)u * N + slot) * D,
                                               q_last + (size_t)u * G * D, G, sM, sL, lane);
            r = (OUT)v;
        }
        if (lane == 0) scores[(size_t)u * N + slot] = r;
    }
}

template <typename OUT> static hipError_t launch_scores_as(const Plan &p, int n, OUT *scores, hipStream_t s)
{
    int chunks = (2048 + p.units - 1) / p.units;
    if (chunks < 1) chunks = 1;
    if (chunks > (p.N + 3) / 4) chunks = (p.N + 3) / 4;
#define LF_SC(T, DD)                                                                            \
    hipLaunchKernelGGL((scores_kernel<T, DD, OUT>), dim3(p.units * chunks), dim3(256), 0, s,    \
                       (const T *)p.k_cache, (const T *)p.v_cache, (const T *)p.q_last, n, p.N, \
                       p.G, p.fin_m, p.fin_l, scores, chunks, p.masked ? p.lu : nullptr, p.ntiles * kTile)
    if (p.dtype == 0) { if (p.D == 64) LF_SC(float, 64); else LF_SC(float, 128); }
    else              { if (p.D == 64) LF_SC(bf16_t, 64); else LF_SC(bf16_t, 128); }
#undef LF_SC
    return hipGetLastError();
}

hipError_t launch_scores(const Plan &p, int n, float *scores, hipStream_t s) { return launch_scores_as(p, n, scores, s); }

// ---------------------------------------------------------------------------------------
// Batch eviction (the every-k-steps regime, Sec. 4.4): one workgroup per unit picks the k
// lowest double-precision scores in ascending (score, slot) order -- round j takes the
// smallest pair above round j-1's, so nothing is written between rounds -- then turns those
// slots, and any not yet filled, into holes of the explicit mask.
// ---------------------------------------------------------------------------------------
template <typename T, int D>
__global__ __launch_bounds__(256) void evict_lowest_kernel(T *__restrict__ Kc, T *__restrict__ Vc,
                                                            const double *__restrict__ sc, float *__restrict__ lu,
                                                            int32_t *__restrict__ pending, int32_t *__restrict__ evicted,
                                                            int n, int N, int k, int lu_stride, int init_lu)
{
    __shared__ double red_v[4];
    __shared__ int red_i[4];
    __shared__ double last_v;
    __shared__ int last_i;
    const int u = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const double *su = sc + (size_t)u * N;
    float *lu_u = lu + (size_t)u * lu_stride;
    if (tid == 0) { last_v = -INFINITY; last_i = -1; }
    // a cache whose kernels never kept the side array (vector-ALU path, prefix mode so far)
    // gets "valid" entries for its filled prefix before the holes are marked
    if (init_lu)
        for (int slot = tid; slot < n; slot += 256) lu_u[(slot & ~15) + tail_pos_of_slot(slot & 15)] = 0.f;
    __syncthreads();
    for (int j = 0; j < k; ++j) {
        const double lv = last_v;
        const int li = last_i;
        double bv = INFINITY;
        int bi = 0x7fffffff;
        for (int i = tid; i < N; i += 256) {
            const double v = su[i]; // +inf marks an invalid slot
            const bool after = v > lv || (v == lv && i > li);
            if (after && v < INFINITY && (v < bv || (v == bv && i < bi))) { bv = v; bi = i; }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            const double ov = __shfl_xor(bv, off);
            const int oi = __shfl_xor(bi, off);
            if (ov < bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
        }
        if (lane == 0) { red_v[wave] = bv; red_i[wave] = bi; }
        __syncthreads();
        if (tid == 0) {
            for (int w = 1; w < 4; ++w)
                if (red_v[w] < bv || (red_v[w] == bv && red_i[w] < bi)) { bv = red_v[w]; bi = red_i[w]; }
            const bool found = bi != 0x7fffffff;
            if (evicted) evicted[(size_t)u * k + j] = found ? bi : -1;
            last_v = found ? bv : INFINITY; // nothing valid is left: later rounds find nothing either
            last_i = found ? bi : 0x7fffffff;
        }
        __syncthreads();
        const int victim = last_i;
        if (victim != 0x7fffffff) { // uniform: the slot becomes a hole with finite (zero) rows
            for (int d = tid; d < D; d += 256) {
                store_elem(Kc + ((size_t)u * N + victim) * D + d, 0.f);
                store_elem(Vc + ((size_t)u * N + victim) * D + d, 0.f);
            }
            if (tid == 0) lu_u[(victim & ~15) + tail_pos_of_slot(victim & 15)] = __builtin_nanf("");
        }
    }
    // slots past a filling cache's prefix become holes of the mask as well
    for (int slot = n + wave; slot < N; slot += 4) {
        for (int d = lane; d < D; d += 64) {
            store_elem(Kc + ((size_t)u * N + slot) * D + d, 0.f);
            store_elem(Vc + ((size_t)u * N + slot) * D + d, 0.f);
        }
        if (lane == 0) lu_u[(slot & ~15) + tail_pos_of_slot(slot & 15)] = __builtin_nanf("");
    }
    __threadfence_block();
    __syncthreads();
    // the next token goes to the lowest hole
    int best = 0x7fffffff;
    for (int p = tid; p < lu_stride; p += 256) {
        const float x = lu_u[p];
        const int slot = (p & ~15) + tail_slot_of_pos(p & 15);
        if (x != x && slot < N) best = min(best, slot);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) best = min(best, __shfl_xor(best, off));
    if (lane == 0) red_i[wave] = best;
    __syncthreads();
    if (tid == 0) {
        best = min(min(red_i[0], red_i[1]), min(red_i[2], red_i[3]));
        if (best != 0x7fffffff) pending[u] = best;
    }
}

hipError_t launch_evict_lowest(const Plan &p, int n, int k, double *scratch, int32_t *evicted, hipStream_t s)
{
    hipError_t e = launch_scores_as(p, n, scratch, s);
    if (e != hipSuccess) return e;
#define LF_EV(T, DD)                                                                             \
    hipLaunchKernelGGL((evict_lowest_kernel<T, DD>), dim3(p.units), dim3(256), 0, s, (T *)p.k_cache, \
                       (T *)p.v_cache, scratch, p.lu, p.pending, evicted, n, p.N, k, p.ntiles * kTile,     \
                       (!p.masked && !p.use_mfma) ? 1 : 0)
    if (p.dtype == 0) { if (p.D == 64) LF_EV(float, 64); else LF_EV(float, 128); }
    else              { if (p.D == 64) LF_EV(bf16_t, 64); else LF_EV(bf16_t, 128); }
#undef LF_EV
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// Score scratch for callers that cannot allocate (longflow_evict_lowest_static): the
// double-precision scores of one batch eviction live in this file-scope device array
// instead of a caller-supplied buffer.  Every GPU the library runs on holds its own copy at
// its own address until the process ends; `scratch` itself is only the host-side stand-in
// for the symbol, never a device address: the address is asked for once per device and kept.
// The score kernel writes every entry the selection kernel reads, so nothing has to be
// cleared between calls; calls that overlap on one GPU would race on it.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) double scratch[kStaticScoreSlots];

hipError_t static_score_scratch(double **ptr)
{
    constexpr int kMaxDevices = 64;
    static double *addr[kMaxDevices] = {};
    static std::mutex mu;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        addr[dev] = (double *)p;
    }
    if (ptr) *ptr = addr[dev];
    return hipSuccess;
}

} // namespace lf
