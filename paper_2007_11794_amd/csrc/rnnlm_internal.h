// Internal declarations shared by the translation units of librnnlm (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>
#include <mutex>

#include "rnnlm.h"
#include "rnnlm_diag.h"

namespace rnnlm {

typedef uint16_t bf16_t;                       // bfloat16 bit pattern

constexpr int kMaxSplits = 256;                // most vocabulary splits of the output projection
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Device-side view of a loaded model (all pointers are device pointers).
struct ModelDev {
    int V, H;
    int Hp;            // H rounded up to a multiple of 64; padded weights are zero
    int Vp;            // V rounded up to a multiple of 256; padded rows of Ot are zero
    int dtype;
    const void *U;     // [V][Hp]
    const void *W;     // [Hp][Hp], W[j][i]
    const void *Ot;    // [Vp][Hp], Ot[v][j] = O[j][v]
    const float *half_rowsum_W;   // [Hp]  0.5 * sum_i W[j][i]
    const float *bias;            // [V]
    const float *half_colsum_O;   // [V]   0.5 * sum_j O[j][v]
    // Additive constant of every base-2 logit, (bias[v] + 0.5*colsum_O[v]) * log2(e); -inf
    // for the padded words v >= V so they add nothing to the sum.
    const float *cvec2;           // [Vp]
    const float *cvec2_fixed;     // [Vp]  cvec2 - m2_fixed
    float m2_fixed;    // upper bound of every base-2 logit z*log2(e), valid because |h' - 0.5| <= 0.5
    // fp32 models with the full softmax: the output projection on the bf16 matrix cores at fp32
    // accuracy.  Every fp32 number is the exact sum of three bf16 numbers x1 + x2 + x3 (8 + 8 + 8
    // mantissa bits); of the nine cross terms of a product the six with the largest weight are
    // kept.  Both operands are kept term-interleaved in chunks of 32 units,
    // [row][unit / 32][term][unit % 32], so a chunk of the reduction is 192 contiguous bytes per row.
    const void *Ot3;   // [Vp][3 Hp] bf16, or null
    // A second copy of the output weights in MFMA-operand order for the kernels that stream them
    // for few rows.  bf16: [Vp / 32][Hp / 16][64 lanes][8], lane 32 g + c of fragment (blk, ks)
    // holds word 32 blk + c, units 16 ks + 8 g .. + 7 (one operand = 1 KB contiguous).  fp32: the
    // same operand as two halves of four floats, [Vp / 32][Hp / 16][2][64 lanes][4].
    const void *Ofrag;
    void *d3;          // [max_Bp][3 Hp] bf16 scratch, or null
    // hierarchical output layer (models loaded with rnnlm_hs_load; Ot .. cvec2_fixed are null then)
    int hs;                       // 1: hierarchical
    const void *Theta;            // [V-1][Hp] node vectors, weights' type, zero-padded
    const int32_t *path_off;      // [V+1]
    const int32_t *path_entry;    // [path_off[V]] node | code bit << 31, root first
    int hs_max_len;               // longest path
    // scratch
    void *d;           // [max_Bp][Hp]  h' - 0.5 in the weights' type
    // bf16 models: the same block times log2(e), in the order the staged output projection reads
    // it, [max_Bp / 32][Hp / 16][64 lanes][8]: lane 32 g + c of fragment (rb, ks) holds row
    // 32 rb + c, units 16 ks + 8 g .. + 7, so one MFMA operand of a wave is 1 KB contiguous.
    void *dfrag;
    float2 *part;      // [max_Bp][kMaxSplits]  (max, sum) partials of the base-2 log-sum-exp
    int *flag;         // sticky rnnlm_device_flag bits
};

// Device-side view of a cache kept between steps (cache.hip).
struct CacheCell {          // one slot of the open-addressing table
    uint64_t key;
    int32_t entry;          // index into the stores, -1 = free
    int32_t pad;
};
struct CacheDev {
    int capacity;           // entries the stores can hold
    int table_size;         // power of two >= 2 * capacity
    int H;
    CacheCell *table;       // [table_size]
    float *store_h;         // [capacity][H]  updated hidden vectors
    float *store_lse;       // [capacity]     natural-log normalisers
    int *n_entries;         // [1]
    long long *totals;      // [4] looked up, found, computed, computed but not kept
    // per-step scratch, each [max_B]
    int32_t *entry_of;      // distinct history u -> its entry (found or newly given), or -1
    int32_t *miss_of;       // u -> row of this step's computed block, or -1 when found
    int32_t *miss_src;      // computed row -> raw query that holds its prev word and h_in
    int32_t *miss_dst;      // computed row -> u
    float *lse_rows;        // [max_B] normaliser of every distinct history of the step
    int *n_miss;            // [1]
    int *block_total;       // [max_B / 1024 + 2] scan scratch of the many-workgroup lookup; last = entries before
};
// Device-side view of an index table (index_table.hip): contexts stored by value, found again
// by content.  The hash table, the counters and the per-call scratch are the cache's.
struct IndexDev {
    CacheDev c;             // c.store_h = hidden vectors [capacity][H]; c.store_lse, c.lse_rows unused
    int32_t *store_word;    // [capacity]
    uint64_t *keys;         // [max_N] content hashes of the call
    int32_t *rep, *inverse; // [max_N] grouping of the call's hashes
    int32_t *n_unique;      // [1]
    void *dedup_ws;
    long long *errors;      // [2] hash collisions caught by the full comparison, bad indices in fetch
};

}  // namespace rnnlm

struct rnnlm_index_table {
    rnnlm::IndexDev dev;
    int max_N;
};

struct rnnlm_cache {
    rnnlm::CacheDev dev;
    int max_B;
};

struct rnnlm_model {
    rnnlm::ModelDev dev;   // the weights' pointers may be another handle's (see owner); the scratch is this handle's
    int max_B, max_Bp;
    int fixed_ok;          // the fixed-offset log-sum-exp is usable for this model
    int lse_mode;          // RNNLM_OPT_LSE_MODE
    int outproj_kernel;    // RNNLM_OPT_OUTPROJ_KERNEL
    hipEvent_t ev0, ev1;
    // Handles made by rnnlm_model_share point at the handle that loaded the weights; that one counts
    // the handles alive on its weights (itself included until it is released) and frees the weights
    // with the last of them.  Both fields are guarded by one library-wide lock.
    rnnlm_model *owner;    // null: this handle loaded the weights
    int handles;           // owner only: handles alive on these weights
    int released;          // owner only: rnnlm_free was called on it, the struct lives on for the others
};

namespace rnnlm {

// A kernel's dynamic-LDS limit, raised once per device to the largest size asked for so far.  Safe
// when two host threads make the first launch at the same time (one static object per kernel).
class LdsLimit {
  public:
    hipError_t ensure(const void *kernel, size_t bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
        if (granted_[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
        std::lock_guard<std::mutex> lock(mutex_);
        if (granted_[dev].load(std::memory_order_relaxed) >= bytes) return hipSuccess;
        e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) granted_[dev].store(bytes, std::memory_order_release);
        return e;
    }

  private:
    static constexpr int kDevices = 64;
    std::mutex mutex_;
    std::atomic<size_t> granted_[kDevices] = {};
};

// ---- launchers (each enqueues on `stream` and returns the hipGetLastError of the launch)

// Grouping of equal 64-bit keys.
size_t dedup_workspace_bytes(int N);
hipError_t launch_dedup(const uint64_t *keys, int N, int32_t *rep, int32_t *inverse,
                        int32_t *n_unique, void *workspace, hipStream_t stream);
// Looks the address of rnnlm_dedup_static's device array up for the current device (status code).
int dedup_static_prepare();

// Hidden update.  rows = number of rows the grid must cover (>= the true B); the true B is
// *B_dev when B_dev != nullptr, else rows.  row_src (nullable) maps row b to the raw row
// that holds its prev word and h_in; row_dst (nullable) maps it to its row of h_out (the
// operand block m.d always takes row b).
hipError_t launch_recur(const ModelDev &m, int rows, const int *B_dev, const int32_t *row_src,
                        const int32_t *row_dst, const int32_t *prev_word, const float *h_in,
                        float *h_out, hipStream_t stream);

constexpr int kStagedRows = 256;   // rows per workgroup of the staged kernel
constexpr int kStagedWords = 32;   // words per LDS stage
constexpr int kXcds = 8;           // workgroup id modulo 8 = the XCD (L2 domain) it runs on

// Work split of an output-projection kernel for B rows on a grid of kXcds * wg_per_xcd workgroups.
// The true B may be known on the device only (after the grouping of ids or the cache lookup), so the
// kernels derive the split there, and the kernels that read the partials afterwards derive the
// same: RG row groups of group_rows rows; the vocabulary is cut into S = kXcds * Sx splits, as
// many as the grid gives every row group (at most sx_cap: one per tile of words); split s is
// served by XCD s % kXcds, so the RG workgroups that stream the same weights share one L2.
struct RowPlan { int RG, Sx, S; };
__host__ __device__ inline RowPlan plan_rows(int B, int group_rows, int wg_per_xcd, int sx_cap) {
    RowPlan p;
    p.RG = (B + group_rows - 1) / group_rows;
    if (p.RG < 1) p.RG = 1;
    p.Sx = wg_per_xcd / p.RG;
    if (p.Sx > sx_cap) p.Sx = sx_cap;
    if (p.Sx > kMaxSplits / kXcds) p.Sx = kMaxSplits / kXcds;
    if (p.Sx < 1) p.Sx = 1;
    p.S = kXcds * p.Sx;
    return p;
}
// First unit of part `index` when `units` units are cut into `parts` nearly equal parts,
// floor(index * units / parts), for 0 <= index <= parts <= 256 and units < 2^31.  With q = units / parts
// and r = units % parts this is index * q + floor(index * r / parts), and index * r stays below 2^16: 32-bit
// arithmetic throughout (a 64-bit division costs a wave some hundred scalar instructions in front of
// its first load).
__host__ __device__ inline int part_begin(int index, int units, int parts) {
    const unsigned q = (unsigned)units / (unsigned)parts, r = (unsigned)units % (unsigned)parts;
    return (int)((unsigned)index * q + ((unsigned)index * r) / (unsigned)parts);
}
typedef RowPlan StagedPlan;
__host__ __device__ inline StagedPlan staged_plan(int B, int wg_per_xcd) {
    return plan_rows(B, kStagedRows, wg_per_xcd, kMaxSplits / kXcds);
}

// How many (max, sum) partials per row the output projection left in m.part: a fixed number, or
// the S of plan_rows for the true number of rows; a kernel that streams the weights when at most
// stream_rows rows are left then leaves one partial per workgroup of its grid.
struct SplitInfo {
    int fixed_splits;      // > 0: that many
    int wg_per_xcd;        // else plan_rows(B, group_rows, wg_per_xcd, sx_cap).S
    int group_rows;
    int sx_cap;
    int stream_rows;       // 0 < B <= stream_rows: kXcds * wg_per_xcd instead
};
__host__ __device__ inline int splits_of(const SplitInfo &si, int B) {
    if (si.fixed_splits > 0) return si.fixed_splits;
    if (B > 0 && B <= si.stream_rows) return kXcds * si.wg_per_xcd;
    return plan_rows(B, si.group_rows, si.wg_per_xcd, si.sx_cap).S;
}
__host__ inline SplitInfo fixed_split_info(int S) { return SplitInfo{S, 0, 1, 1, 0}; }

// Output projection + log-sum-exp partials over the vocabulary, on the block m.d.
hipError_t launch_outproj(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                          int kernel_choice, SplitInfo *splits, hipStream_t stream);
// false: the kernel launch_outproj takes for these arguments reads only the fragment-ordered copy of
// the hidden block, and the hidden update may leave the row-ordered one (m.d) unwritten
bool outproj_reads_row_order(const ModelDev &m, int rows, bool fixed_offset, int kernel_choice);
const char *outproj_kernel_name(const ModelDev &m, int rows, bool fixed_offset, int kernel_choice);
bool outproj_staged_supported(const ModelDev &m);
bool outproj_rowstream_supported(const ModelDev &m);   // bf16 models
int outproj_stream_max_rows(const ModelDev &m);   // 0: the weight-streaming kernel cannot serve this model

// Query gather: logprob[n][k] = z[row(n)][query[n][k]] - lse[row(n)] - base_score[n][k].
// lse comes from lse_rows[row] when that is given, else from the partials in m.part;
// base_score may be null.
hipError_t launch_query(const ModelDev &m, int rows, const int *B_dev, int N, int K, SplitInfo splits,
                        const int32_t *query_word, const int32_t *row_of_query,
                        const float *h_out, const float *lse_rows, const float *base_score,
                        float *logprob, hipStream_t stream);

// The same through a cache (after launch_cache_lookup and the computation of the histories not
// found): found histories take h' and lse from the stores, and the first raw query of every distinct
// history passes its h' on (to h_out when found, into the store with its lse when it got an entry),
// which is all that launch_cache_commit does otherwise.  rows / n_unique: distinct histories.
hipError_t launch_query_cached(const ModelDev &m, const CacheDev &c, int rows, const int32_t *n_unique, int N, int K,
                               SplitInfo splits, const int32_t *query_word, const int32_t *inverse,
                               const int32_t *rep, float *h_out, const float *base_score, float *score,
                               hipStream_t stream);

// ---- cache kept between steps (cache.hip)
hipError_t launch_cache_reset(const CacheDev &c, hipStream_t stream);
// Looks the distinct histories ids[rep[u]], u < *n_unique, up; numbers the ones not found
// (in order of u), gives them entries while there is room and inserts their keys.
// rows = upper bound of *n_unique (sizes the grid).  Up to one_group_rows the lookup is one launch
// of one workgroup (best while the table sits in L2: the step's cache, up to 4096), beyond it
// three launches of a full grid (best when the probes go to HBM: the index table, from 1024).
hipError_t launch_cache_lookup(const CacheDev &c, int rows, int one_group_rows, const uint64_t *ids,
                               const int32_t *rep, const int32_t *n_unique, int32_t *step_stats,
                               hipStream_t stream);
// Grouping of the ids (launch_dedup) and this lookup in ONE launch of one workgroup, for
// 0 < N <= dedup_lookup_max_rows() raw queries.
int dedup_lookup_max_rows();
hipError_t launch_dedup_lookup(const CacheDev &c, const uint64_t *ids, int N, int32_t *rep, int32_t *inverse,
                               int32_t *n_unique, int32_t *step_stats, hipStream_t stream);
// After the computed block is done: normalisers of all distinct histories into c.lse_rows,
// new entries into the stores, stored hidden vectors of found histories into h_out.
hipError_t launch_cache_commit(const CacheDev &c, const ModelDev &m, int rows, const int32_t *n_unique,
                               SplitInfo splits, float *h_out, hipStream_t stream);
// Index table: content hashes of N contexts; after grouping and lookup, storage of the new
// contexts, full comparison of every context with the one it was identified with, and the
// indices; gather of stored contexts.
hipError_t launch_index_reset(const IndexDev &t, hipStream_t stream);
hipError_t launch_context_hash(const int32_t *word, const float *h, int N, int H, uint64_t *keys,
                               hipStream_t stream);
hipError_t launch_index_commit(const IndexDev &t, int N, const int32_t *word, const float *h, uint32_t *index,
                               hipStream_t stream);
hipError_t launch_index_fetch(const IndexDev &t, int N, const uint32_t *index, int32_t *word, float *h,
                              hipStream_t stream);
// Hierarchical output layer: logprob[n][k] = sum over the path of query[n][k] of
// log sigmoid(+-theta_node . h'[row(n)]) (- base_score[n][k]).
hipError_t launch_hs_query(const ModelDev &m, int rows, const int *B_dev, int N, int K,
                           const int32_t *query_word, const int32_t *row_of_query, const float *h_out,
                           const float *base_score, float *logprob, hipStream_t stream);
hipError_t launch_pack_ids(const uint32_t *ctx, const uint32_t *small_lm, int N, uint64_t *ids,
                           hipStream_t stream);

// Load-time helpers.
hipError_t launch_transpose_O(const void *O_dev /*[H][V]*/, void *Ot /*[Vp][Hp]*/, int dtype,
                              int H, int V, int Hp, int Vp, hipStream_t stream);
hipError_t launch_col_stats(const void *O_dev, const float *bias_or_null, int dtype, int H, int V,
                            float *half_colsum /*[V]*/, float *upper /*[V]*/, float *lower /*[V]*/,
                            hipStream_t stream);
hipError_t launch_frag_weights(const void *Ot /*[Vp][Hp]*/, int dtype, int Vp, int Hp, void *Ofrag, hipStream_t stream);
hipError_t launch_split3_weights(const float *Ot /*[Vp][Hp]*/, int Vp, int Hp, void *Ot3 /*[Vp][3 Hp] bf16*/,
                                 hipStream_t stream);
hipError_t launch_fill_cvec(const float *bias_or_null, const float *half_colsum, int V, int Vp,
                            float m2_fixed, float *bias_out, float *cvec2, float *cvec2_fixed,
                            hipStream_t stream);

}  // namespace rnnlm
