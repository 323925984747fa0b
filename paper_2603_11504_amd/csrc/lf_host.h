// Internal host-side declarations shared by the C-ABI layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace lf {

constexpr int kTile = 16;      // slots per screening-stash tile (one MFMA tile of slots)
constexpr int kMaxSplits = 64; // upper bound on split-K factor
constexpr int kMaxGroup = 16;  // query heads per KV head
// dynamic LDS the unit-resident kernel may ask for: 160 KB per CU minus its static part
constexpr size_t kUnitLdsLimit = 160 * 1024 - 12 * 1024;

// Everything a launch needs; filled by the API layer.
struct Plan {
    int B, Hq, Hkv, D, N, G, units;
    int dtype;         // 0 = f32, 1 = bf16
    uint32_t flags;
    int L;             // slots per split (multiple of kTile)
    int C;             // number of splits covering N
    int ntiles;        // ceil(N / kTile)
    bool use_mfma;     // bf16, head_dim 128: matrix-core kernels
    bool use_mfma32;   // fp32, or bf16 with head_dim 64: split-K kernel on the matrix cores in fp32 arithmetic
    bool use_unit;     // unit-resident fused kernel: whole step in one launch
    int unit_S;        // ... with this many cooperating workgroups per unit
    bool masked;       // an explicit validity mask is in force (state, set by longflow_set_mask)
    bool unfused;      // comparison path: plain attention kernel, then separate importance kernels
    bool max_free;     // softmax without a running reference, as Alg. 1 prints it (A/B measurement)
    // device pointers (caller-owned)
    void *k_cache, *v_cache;
    // carved out of the caller's workspace
    int32_t *pending;  // [units]
    int32_t *arrive;   // [units] arrival counters of cooperating workgroups, zero between steps
    void *q_last;      // [B][Hq][D] copy of the last step's query (for longflow_scores)
    float *part_m;     // [units][C][G]    split-local softmax reference (log2 domain)
    float *part_l;     // [units][C][G]    split-local denominator
    float *part_o;     // [units][C][G][D] split-local un-normalised output
    float *fin_m;      // [units][G]       global reference of the last step
    float *fin_l;      // [units][G]       global denominator of the last step
    uint16_t *stash_w; // [units][ntiles][G][kTile] bf16 screening values ||v||_1 * p
    float *stash_m;    // [units][ntiles][G]        reference each tile's p is relative to
    float *lu;         // [units][ntiles*kTile] log2 ||v||_1 per slot, position order inside a tile
                       // (kept current by init and insert; NaN = slot invalid under an explicit
                       // mask; the vector-ALU kernels use it for validity only)
    int32_t *first_hole; // [units] scratch of the mask setter
    // comparison path only
    float *acc;          // [units][ntiles*kTile] attention weight received since insertion (position order)
    float *acc_part_v;   // [units][CA] lowest accumulator of each span ...
    int32_t *acc_part_i; // [units][CA] ... and its slot
};

struct Layout {
    size_t off_pending, off_arrive, off_hole, off_q, off_part_m, off_part_l, off_part_o, off_fin_m, off_fin_l,
        off_stash_w, off_stash_m, off_lu, off_acc, off_acc_part_v, off_acc_part_i, total;
    // the same carving as a list (name, offset, bytes asked for), in order: longflow_workspace_regions
    static constexpr int kMaxRegions = 24;
    int n_regions;
    const char *region_name[kMaxRegions];
    size_t region_off[kMaxRegions], region_bytes[kMaxRegions];
};

// Split-K geometry for a cache of `units` independent (batch, KV head) pairs.
void choose_splits(int units, int N, int *L, int *C);

// Kernel launchers (each returns the hipError_t of its launch).
// One decode step on a split-K path (single launch: insert, stream, last-arriver finish).
struct StepIo {
    const void *q, *k_new, *v_new;
    void *out;
    int32_t *evict_idx;
};
// table/n_caches: several caches in one grid (see split_table_entry); nullptr/1 = one cache
hipError_t launch_split_valu(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table = nullptr,
                             int n_caches = 1);
hipError_t launch_split_mfma(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table = nullptr,
                             int n_caches = 1);
hipError_t launch_split_mfma32(const Plan &p, const StepIo &io, int n, hipStream_t s, const void *table = nullptr,
                               int n_caches = 1);
size_t split_table_entry_bytes();
void split_table_entry(const Plan &p, void *dst);
int unit_mfma_splits(int units, int N);
int unit_mfma_split_len(int N, int S);
size_t unit_mfma_lds_bytes(int N, int G, bool stash, int S);
hipError_t launch_unit_mfma(const Plan &p, const void *q, const void *k_new, const void *v_new, int n,
                            void *out, int32_t *evict_idx, hipStream_t s);
// Several caches of one geometry in one grid: `table` is a device array with one entry
// (unit_mfma_table_entry_bytes() each, written by unit_mfma_table_entry on the host and
// copied over) per cache; io holds base pointers, cache i's tensors follow at i times the
// tensor's size.
size_t unit_mfma_table_entry_bytes();
void unit_mfma_table_entry(const Plan &p, void *dst);
hipError_t launch_unit_mfma_group(const Plan &p, const StepIo &io, int n, const void *table, int n_caches,
                                  hipStream_t s);
// Comparison path (accumulated attention weights): insert, plain attention, accumulate, decide.
void unfused_geometry(int units, int N, int *LA, int *CA);
hipError_t launch_unfused_step(const Plan &p, const StepIo &io, int n, hipStream_t s);
hipError_t launch_unfused_scores(const Plan &p, float *scores, hipStream_t s); // float [units][N]
// Fill phase in bulk (bf16, head_dim 128): rows n0 .. n0 + Tb - 1 from k_new / v_new ([Tb][units][128]), then
// causal attention of the Tb queries ([Tb][units][G][128]) -> out, fill_tokens_per_pass(G) tokens per pass over the cache.
int fill_tokens_per_pass(int G);
hipError_t launch_fill_bulk(const Plan &p, const void *q, const void *k_new, const void *v_new, void *out, int n0,
                            int Tb, hipStream_t s);
// One-shot compression of a prompt of T rows to `keep` rows (observation window of W rows, votes pooled over
// `pool` rows): fills slots [0, keep) of the cache and its side array.  Scratch as carved by compress_layout
// (keep_max = the cache's budget); pooled votes float [units][T - W] and kept rows int32 [units][keep] stay there.
struct CompressLayout {
    size_t off_part_m, off_part_l, off_cq, off_votes, off_pooled, off_kept, total;
};
void compress_geometry(int units, int T, int *LS, int *nspans);
CompressLayout compress_layout(int units, int G, int T, int W, int keep_max);
hipError_t launch_compress_prompt(const Plan &p, int T, int W, int keep, int pool, const void *q_window,
                                  const void *k_prompt, const void *v_prompt, void *scratch, hipStream_t s);
hipError_t launch_scores(const Plan &p, int n, float *scores, hipStream_t s);
// Drop the k lowest-scoring valid slots of every unit (scores of the last step, in double
// precision via `scratch`, device double [units][N]); they become holes of the explicit mask.
hipError_t launch_evict_lowest(const Plan &p, int n, int k, double *scratch, int32_t *evicted, hipStream_t s);
// Batch eviction without a caller-supplied scratch buffer: a file-scope device array of
// kStaticScoreSlots doubles (one per slot of the cache) stands in.  static_score_scratch
// resolves its address on the current device (once per device; later calls are a table
// look-up) and stores it in *ptr if ptr is not null.
constexpr size_t kStaticScoreSlots = (size_t)1 << 20; // 8 MiB per GPU
hipError_t static_score_scratch(double **ptr);
hipError_t launch_l1norms(const Plan &p, int n_rows, hipStream_t s);
hipError_t launch_fill_i32(int32_t *dst, int count, int32_t value, hipStream_t s);
// A group's table entry (at most kTableEntryMax bytes, a multiple of 4) travels to dst as a kernel
// argument: no host buffer has to outlive the call and nothing synchronises with the host.
constexpr size_t kTableEntryMax = 256;
hipError_t launch_table_entry(void *dst, const void *entry, size_t bytes, hipStream_t s);
// Explicit mask (device uint8 [units][N], nonzero = valid): rewrites the side array, zeroes
// the K/V rows of invalid slots and points `pending` of every unit that has an invalid
// slot at its lowest one.
hipError_t launch_set_mask(const Plan &p, const uint8_t *mask, hipStream_t s);
hipError_t launch_get_mask(const Plan &p, int n, uint8_t *mask, hipStream_t s);

} // namespace lf
