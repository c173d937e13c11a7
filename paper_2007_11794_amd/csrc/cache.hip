// The cache of RnnlmProb kept on the device between steps (Table 1 as a whole; Section 4.2:
// once-computed results are reused for the same context; Section 5.3: a size boundary).
//
// Key: the 8-byte history id (Section 3.2).  Value: what every answer for that history is
// made of -- its updated hidden vector h' (fp32) and its natural-log normaliser -- so a
// history found here skips the hidden update and the whole-vocabulary normalisation; only
// the H-long dot products of its queried words remain.  Entries are numbered in the order
// in which they were stored (Table 1 step 10) and never removed; the table is open
// addressing over 16-byte cells, at most half full.
//
// One step through the cache, after the grouping of the step's own ids:
//   lookup   probe every distinct history; the ones not found are numbered in order of
//            appearance by a prefix sum (row of the block that is computed now), get the next
//            entries while there is room, and their keys are inserted.  One workgroup in one
//            launch for few histories, three launches of a full grid (probe + counts, scan of
//            the counts, numbering + insertion) for many;
//   (hidden update and output projection run on the numbered rows only)
//   commit   per distinct history: normaliser into lse_rows; new entries are written to the
//            stores, found ones copy their stored h' to the caller's h_out.
#include "dedup_small_body.h"
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kLookupThreads = 1024;

__global__ __launch_bounds__(256) void cache_reset_kernel(CacheDev c) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < c.table_size) {
        CacheCell cell;
        cell.key = 0;
        cell.entry = -1;
        cell.pad = 0;
        c.table[i] = cell;
    }
    if (i == 0) *c.n_entries = 0;
    if (i < 4) c.totals[i] = 0;
}

// One workgroup.  A round covers kLookupPer * 1024 distinct histories: every thread first
// requests the first table cell of all its kLookupPer histories (the usual probe ends there),
// then finishes the probes, then the round's misses are numbered chunk by chunk in order of
// u, and last the new keys are inserted.  Insertions happen only after every probe of the
// round is over (barriers of the scans in between), so no probe reads a half-written cell;
// the keys of one step are distinct, so a later round can never look for a key that an
// earlier round of the same step inserted.
constexpr int kLookupPer = 4;

// raw_of(u0, i, u) / key_of(u0, i, u, raw): representative and id of distinct history u (slice i of
// the round that starts at u0), u < U.
template <typename RawOf, typename KeyOf>
__device__ __forceinline__ void cache_lookup_body(const CacheDev &c, int U, int32_t *__restrict__ step_stats,
                                                  RawOf raw_of, KeyOf key_of) {
    __shared__ int wsum[kLookupThreads / 64 + 1];
    const int base = *c.n_entries;          // read by everyone before thread 0 updates it below
    const uint32_t mask = (uint32_t)(c.table_size - 1);
    int n_miss = 0;                         // misses numbered so far (same in every thread)
    for (int u0 = 0; u0 < U; u0 += kLookupPer * kLookupThreads) {
        uint64_t key[kLookupPer];
        int raw[kLookupPer], found[kLookupPer];
        uint32_t h[kLookupPer];
        CacheCell cell[kLookupPer];
#pragma unroll
        for (int i = 0; i < kLookupPer; ++i) {
            const int u = u0 + i * kLookupThreads + (int)threadIdx.x;
            raw[i] = (u < U) ? raw_of(u0, i, u) : 0;
        }
#pragma unroll
        for (int i = 0; i < kLookupPer; ++i) {
            const int u = u0 + i * kLookupThreads + (int)threadIdx.x;
            key[i] = (u < U) ? key_of(u0, i, u, raw[i]) : 0;
            h[i] = mix64(key[i]) & mask;
            cell[i] = c.table[h[i]];
        }
#pragma unroll
        for (int i = 0; i < kLookupPer; ++i) {
            found[i] = -1;
            // At most capacity <= table_size / 2 cells are taken: a free cell is always met.
            for (int probe = 0; probe < c.table_size; ++probe) {
                if (cell[i].entry < 0) break;
                if (cell[i].key == key[i]) { found[i] = cell[i].entry; break; }
                h[i] = (h[i] + 1) & mask;
                cell[i] = c.table[h[i]];
            }
        }
        int entry[kLookupPer];
#pragma unroll
        for (int i = 0; i < kLookupPer; ++i) {
            const int u = u0 + i * kLookupThreads + (int)threadIdx.x;
            entry[i] = -1;
            if (u0 + i * kLookupThreads >= U) continue;       // uniform: nobody has a history in this slice
            const bool active = u < U;
            const int miss = (active && found[i] < 0) ? 1 : 0;
            int total;
            const int rank = n_miss + block_exclusive_scan(miss, wsum, total);
            n_miss += total;
            entry[i] = -1;
            if (miss) {
                entry[i] = (base + rank < c.capacity) ? base + rank : -1;
                c.miss_of[u] = rank;
                c.miss_src[rank] = raw[i];
                c.miss_dst[rank] = u;
                c.entry_of[u] = entry[i];
            } else if (active) {
                c.miss_of[u] = -1;
                c.entry_of[u] = found[i];
            }
        }
        // every probe of this round is done (the scans above contain barriers)
#pragma unroll
        for (int i = 0; i < kLookupPer; ++i) {
            if (entry[i] < 0) continue;
            uint32_t hh = mix64(key[i]) & mask;
            for (int probe = 0; probe < c.table_size; ++probe) {
                if (atomicCAS(&c.table[hh].entry, -1, entry[i]) == -1) {
                    c.table[hh].key = key[i];
                    break;
                }
                hh = (hh + 1) & mask;
            }
        }
        __threadfence_block();
        __syncthreads();                    // this round's insertions precede the next round's probes
    }
    if (threadIdx.x == 0) {
        const int stored = min(n_miss, max(c.capacity - base, 0));
        *c.n_miss = n_miss;
        *c.n_entries = base + stored;
        c.totals[0] += U;
        c.totals[1] += U - n_miss;
        c.totals[2] += n_miss;
        c.totals[3] += n_miss - stored;
        if (step_stats) {
            step_stats[0] = U;
            step_stats[1] = U - n_miss;
            step_stats[2] = n_miss;
            step_stats[3] = base + stored;
        }
    }
}

__global__ __launch_bounds__(kLookupThreads) void cache_lookup_kernel(
    CacheDev c, int rows, const uint64_t *__restrict__ ids, const int32_t *__restrict__ rep,
    const int32_t *__restrict__ n_unique, int32_t *__restrict__ step_stats) {
    // The first slice's representatives and ids are requested before the number of distinct
    // histories is known (rep has `rows` slots; what lies beyond the true count is clamped into
    // range and dropped later): one memory latency less at the head of the chain.
    const int u_first = (int)threadIdx.x;
    int raw_first = (u_first < rows) ? rep[u_first] : 0;
    raw_first = max(min(raw_first, rows - 1), 0);
    const uint64_t key_first = (rows > 0) ? ids[raw_first] : 0;
    const int U = *n_unique;
    cache_lookup_body(
        c, U, step_stats, [&](int u0, int i, int u) { return (u0 == 0 && i == 0) ? raw_first : rep[u]; },
        [&](int u0, int i, int u, int raw) { return (u0 == 0 && i == 0) ? key_first : ids[raw]; });
}

// Grouping of the step's ids and the lookup of the distinct ones in one launch of one workgroup
// (N <= kSmallN): the lookup takes representatives and ids from LDS, where the grouping left them,
// so nothing is read back from memory between the two and one launch is saved.
static_assert(kLookupThreads == kSmallThreads, "");
__global__ __launch_bounds__(kLookupThreads) void dedup_lookup_kernel(
    CacheDev c, const uint64_t *__restrict__ ids, int N, int32_t *__restrict__ rep,
    int32_t *__restrict__ inverse, int32_t *__restrict__ n_unique, int32_t *__restrict__ step_stats) {
    const SmallGroups g = dedup_small_body(ids, N, rep, inverse, n_unique);
    __syncthreads();                        // the groups in LDS are complete
    cache_lookup_body(
        c, g.total, step_stats, [&](int, int, int u) { return g.rep[u]; },
        [&](int, int, int u, int) { return g.id[u]; });
}

// The same for up to kMediumN raw queries (the grouping keeps the keys in LDS in raw order).
__global__ __launch_bounds__(kLookupThreads) void dedup_lookup_medium_kernel(
    CacheDev c, const uint64_t *__restrict__ ids, int N, int32_t *__restrict__ rep,
    int32_t *__restrict__ inverse, int32_t *__restrict__ n_unique, int32_t *__restrict__ step_stats) {
    const MediumGroups g = dedup_medium_body(ids, N, rep, inverse, n_unique);
    __syncthreads();                        // the representatives in LDS are complete
    cache_lookup_body(
        c, g.total, step_stats, [&](int, int, int u) { return g.rep[u]; },
        [&](int, int, int, int raw) { return g.key[raw]; });
}

// ---- the same lookup for many histories (more than one workgroup can number in one round):
// probe + per-workgroup miss counts, a scan of the counts, then numbering + insertion.  The
// launch boundaries put every probe before every insertion.
__device__ __forceinline__ int probe_table(const CacheDev &c, uint64_t key) {
    const uint32_t mask = (uint32_t)(c.table_size - 1);
    uint32_t h = mix64(key) & mask;
    for (int probe = 0; probe < c.table_size; ++probe) {
        const CacheCell cell = c.table[h];
        if (cell.entry < 0) return -1;
        if (cell.key == key) return cell.entry;
        h = (h + 1) & mask;
    }
    return -1;
}

__global__ __launch_bounds__(kLookupThreads) void lookup_probe_kernel(
    CacheDev c, const uint64_t *__restrict__ ids, const int32_t *__restrict__ rep,
    const int32_t *__restrict__ n_unique) {
    __shared__ int wsum[kLookupThreads / 64 + 1];
    const int U = *n_unique;
    const int u = blockIdx.x * kLookupThreads + (int)threadIdx.x;
    int miss = 0;
    if (u < U) {
        const int found = probe_table(c, ids[rep[u]]);
        c.entry_of[u] = found;
        miss = found < 0 ? 1 : 0;
    }
    int total;
    (void)block_exclusive_scan(miss, wsum, total);
    if (threadIdx.x == 0) c.block_total[blockIdx.x] = total;
}

__global__ __launch_bounds__(kLookupThreads) void lookup_scan_kernel(CacheDev c, int blocks,
                                                                     const int32_t *__restrict__ n_unique,
                                                                     int32_t *__restrict__ step_stats) {
    __shared__ int wsum[kLookupThreads / 64 + 1];
    int carry = 0;
    for (int b0 = 0; b0 < blocks; b0 += kLookupThreads) {
        const int b = b0 + (int)threadIdx.x;
        const int v = (b < blocks) ? c.block_total[b] : 0;
        int total;
        const int excl = carry + block_exclusive_scan(v, wsum, total);
        if (b < blocks) c.block_total[b] = excl;
        carry += total;
    }
    if (threadIdx.x == 0) {
        const int U = *n_unique, n_miss = carry, base = *c.n_entries;
        const int stored = min(n_miss, max(c.capacity - base, 0));
        c.block_total[blocks] = base;               // entries before this call, for the numbering
        *c.n_miss = n_miss;
        *c.n_entries = base + stored;
        c.totals[0] += U;
        c.totals[1] += U - n_miss;
        c.totals[2] += n_miss;
        c.totals[3] += n_miss - stored;
        if (step_stats) {
            step_stats[0] = U;
            step_stats[1] = U - n_miss;
            step_stats[2] = n_miss;
            step_stats[3] = base + stored;
        }
    }
}

__global__ __launch_bounds__(kLookupThreads) void lookup_assign_kernel(
    CacheDev c, int blocks, const uint64_t *__restrict__ ids, const int32_t *__restrict__ rep,
    const int32_t *__restrict__ n_unique) {
    __shared__ int wsum[kLookupThreads / 64 + 1];
    const int U = *n_unique;
    const int base = c.block_total[blocks];
    const int u = blockIdx.x * kLookupThreads + (int)threadIdx.x;
    const bool active = u < U;
    const int miss = (active && c.entry_of[u] < 0) ? 1 : 0;
    int total;
    const int rank = c.block_total[blockIdx.x] + block_exclusive_scan(miss, wsum, total);
    if (miss) {
        const int raw = rep[u];
        const uint64_t key = ids[raw];
        const int entry = (base + rank < c.capacity) ? base + rank : -1;
        c.miss_of[u] = rank;
        c.miss_src[rank] = raw;
        c.miss_dst[rank] = u;
        c.entry_of[u] = entry;
        if (entry >= 0) {
            const uint32_t mask = (uint32_t)(c.table_size - 1);
            uint32_t h = mix64(key) & mask;
            for (int probe = 0; probe < c.table_size; ++probe) {
                if (atomicCAS(&c.table[h].entry, -1, entry) == -1) {
                    c.table[h].key = key;
                    break;
                }
                h = (h + 1) & mask;
            }
        }
    } else if (active) {
        c.miss_of[u] = -1;
    }
}

__global__ __launch_bounds__(256) void cache_commit_kernel(CacheDev c, ModelDev m,
                                                            const int32_t *__restrict__ n_unique,
                                                            SplitInfo si, float *__restrict__ h_out) {
    const int u = blockIdx.x;
    if (u >= *n_unique) return;
    const int H = c.H;
    const int row = c.miss_of[u], entry = c.entry_of[u];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    float *hrow = h_out + (size_t)u * H;
    if (row >= 0) {
        // computed in this step: its partials are in row `row` of the block of *n_miss rows
        // (a model with the hierarchical output layer has no normaliser: the hidden vector is all)
        if (wave == 0 && !m.hs) {
            const int splits = splits_of(si, *c.n_miss);
            const float lse = lse_from_partials(m.part + (size_t)row * kMaxSplits, splits, lane);
            if (lane == 0) {
                c.lse_rows[u] = lse;
                if (entry >= 0) c.store_lse[entry] = lse;
            }
        }
        if (entry >= 0) {
            float *dst = c.store_h + (size_t)entry * H;
            for (int j = threadIdx.x; j < H; j += 256) dst[j] = hrow[j];
        }
    } else {
        const float *src = c.store_h + (size_t)entry * H;
        for (int j = threadIdx.x; j < H; j += 256) hrow[j] = src[j];
        if (threadIdx.x == 0 && !m.hs) c.lse_rows[u] = c.store_lse[entry];
    }
}

__global__ __launch_bounds__(256) void pack_ids_kernel(const uint32_t *__restrict__ ctx,
                                                        const uint32_t *__restrict__ small_lm, int N,
                                                        uint64_t *__restrict__ ids) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    if (n < N) ids[n] = ((uint64_t)ctx[n] << 32) | (uint64_t)small_lm[n];
}

}  // namespace

hipError_t launch_cache_reset(const CacheDev &c, hipStream_t stream) {
    const int n = c.table_size > 4 ? c.table_size : 4;
    hipLaunchKernelGGL(cache_reset_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, c);
    return hipGetLastError();
}

hipError_t launch_cache_lookup(const CacheDev &c, int rows, int one_group_rows, const uint64_t *ids,
                               const int32_t *rep, const int32_t *n_unique, int32_t *step_stats,
                               hipStream_t stream) {
    if (rows <= one_group_rows) {                       // few histories: one workgroup, one launch
        hipLaunchKernelGGL(cache_lookup_kernel, dim3(1), dim3(kLookupThreads), 0, stream, c, rows, ids, rep, n_unique,
                           step_stats);
        return hipGetLastError();
    }
    const int blocks = (rows + kLookupThreads - 1) / kLookupThreads;
    hipLaunchKernelGGL(lookup_probe_kernel, dim3(blocks), dim3(kLookupThreads), 0, stream, c, ids, rep, n_unique);
    hipLaunchKernelGGL(lookup_scan_kernel, dim3(1), dim3(kLookupThreads), 0, stream, c, blocks, n_unique,
                       step_stats);
    hipLaunchKernelGGL(lookup_assign_kernel, dim3(blocks), dim3(kLookupThreads), 0, stream, c, blocks, ids, rep,
                       n_unique);
    return hipGetLastError();
}

int dedup_lookup_max_rows() { return kMediumN; }

hipError_t launch_dedup_lookup(const CacheDev &c, const uint64_t *ids, int N, int32_t *rep, int32_t *inverse,
                               int32_t *n_unique, int32_t *step_stats, hipStream_t stream) {
    if (N <= 0 || N > kMediumN) return hipErrorInvalidValue;
    if (N <= kSmallN)
        hipLaunchKernelGGL(dedup_lookup_kernel, dim3(1), dim3(kLookupThreads), 0, stream, c, ids, N, rep, inverse,
                           n_unique, step_stats);
    else
        hipLaunchKernelGGL(dedup_lookup_medium_kernel, dim3(1), dim3(kLookupThreads), 0, stream, c, ids, N, rep,
                           inverse, n_unique, step_stats);
    return hipGetLastError();
}

hipError_t launch_cache_commit(const CacheDev &c, const ModelDev &m, int rows, const int32_t *n_unique,
                               SplitInfo splits, float *h_out, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(cache_commit_kernel, dim3(rows), dim3(256), 0, stream, c, m, n_unique, splits, h_out);
    return hipGetLastError();
}

hipError_t launch_pack_ids(const uint32_t *ctx, const uint32_t *small_lm, int N, uint64_t *ids,
                           hipStream_t stream) {
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(pack_ids_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, ctx, small_lm, N, ids);
    return hipGetLastError();
}

}  // namespace rnnlm
