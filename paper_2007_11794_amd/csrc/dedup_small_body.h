// The one-workgroup grouping of history ids (N <= kSmallN, and a second form up to kMediumN) as device functions: the kernel of its
// own runs it, and so does the kernel that goes on to the cache lookup in the same launch.
#pragma once

#include "device_utils.h"

namespace rnnlm {

constexpr uint64_t kEmpty = 0xFFFFFFFFFFFFFFFFull;   // marks a free slot; the key with this
                                                     // value lives in a slot of its own
constexpr int kSmallN = 4096;
constexpr int kSmallCap = 8192;                      // LDS slots of the small path
constexpr int kSmallThreads = 1024;

// Find or claim the slot of `key` in an open-addressing table of `cap` slots (+1 extra slot
// at index cap for the key that equals the free marker).
template <typename KeyPtr>
__device__ __forceinline__ int find_or_insert(KeyPtr tkeys, int cap, uint64_t key) {
    if (key == kEmpty) return cap;
    uint32_t h = mix64(key) & (uint32_t)(cap - 1);
    // The table holds at most N <= cap/2 keys, so a free slot is always met.
    for (int probe = 0; probe < cap; ++probe) {
        unsigned long long old = atomicCAS(reinterpret_cast<unsigned long long *>(&tkeys[h]),
                                           (unsigned long long)kEmpty, (unsigned long long)key);
        if (old == kEmpty || old == key) return (int)h;
        h = (h + 1) & (uint32_t)(cap - 1);
    }
    return -1;   // unreachable for N <= cap/2
}

// What the grouping leaves in LDS for a consumer in the same workgroup (valid after a barrier):
// representative and id of group u < total.  The arrays lie in the key table, which is free by then.
struct SmallGroups {
    int total;
    const int *rep;          // [total]
    const uint64_t *id;      // [total]
};

// All kSmallThreads threads of the one workgroup call it; N <= kSmallN.
__device__ __forceinline__ SmallGroups dedup_small_body(const uint64_t *__restrict__ keys, int N,
                                                        int32_t *__restrict__ rep, int32_t *__restrict__ inverse,
                                                        int32_t *__restrict__ n_unique) {
    __shared__ uint64_t tkeys[kSmallCap + 1];
    __shared__ int tfirst[kSmallCap + 1];    // min raw index per slot, later the group number
    __shared__ int wsum[kSmallThreads / 64 + 1];
    constexpr int kPer = kSmallN / kSmallThreads;      // queries per thread
    static_assert(kSmallN * 4 + kSmallN * 8 <= kSmallCap * 8, "rep and id of every group fit the key table");
    int *const rep_lds = reinterpret_cast<int *>(tkeys);                 // [kSmallN] ints = kSmallN / 2 slots
    uint64_t *const id_lds = tkeys + kSmallN / 2;                        // [kSmallN]

    // Thread t owns the `per` contiguous queries from t * per on (per = ceil(N / threads), so all
    // threads take part whatever N is); contiguous ownership makes the scan below run over
    // raw-index order.  The keys are fetched first, all at once: an insertion is a loop around an
    // LDS atomic, and a load behind it would wait for it.
    const int per = (N + kSmallThreads - 1) / kSmallThreads;
    uint64_t key[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        key[i] = (i < per && n < N) ? keys[n] : 0;
    }
    for (int i = threadIdx.x; i <= kSmallCap; i += kSmallThreads) {     // while the keys are on their way
        tkeys[i] = kEmpty;
        tfirst[i] = 0x7FFFFFFF;
    }
    __syncthreads();
    int slot[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        slot[i] = -1;
        if (i < per && n < N) {
            slot[i] = find_or_insert(tkeys, kSmallCap, key[i]);
            atomicMin(&tfirst[slot[i]], n);
        }
    }
    __syncthreads();

    int is_first[kPer];
    int mine = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        int n = threadIdx.x * per + i;
        is_first[i] = (slot[i] >= 0 && tfirst[slot[i]] == n) ? 1 : 0;
        mine += is_first[i];
    }
    int total;
    int u = block_exclusive_scan(mine, wsum, total);   // barriers inside: all tfirst reads done
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        if (is_first[i]) {
            int n = threadIdx.x * per + i;
            rep[u] = n;
            rep_lds[u] = n;                            // (the key table is not read any more)
            id_lds[u] = key[i];
            tfirst[slot[i]] = u;                       // the slot now carries its group number
            ++u;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        int n = threadIdx.x * per + i;
        if (slot[i] >= 0) inverse[n] = tfirst[slot[i]];
    }
    if (threadIdx.x == 0) *n_unique = total;
    return SmallGroups{total, rep_lds, id_lds};
}

// ------------------------------------------------------------------------------ up to kMediumN ids
// The same grouping for more ids in the same LDS: the table keeps, per slot, the
// index of a raw query (4 bytes) instead of the key (8 bytes), and the keys themselves sit in LDS
// once, in raw order; a probe compares its key with the key of the query the slot points to.  A
// slot's index is only ever replaced by a smaller index of the SAME key (atomicMin after the
// comparison), so the key a slot stands for never changes, and after all insertions the slot holds
// the first raw index of its group.  No key value is special here.
// (7 ids per thread; with 8192 ids, half of the slots taken, the probe chains make the one workgroup
// slower than the launches of the grid-wide form: 16 to 30 us against 18 to 20, measured)
constexpr int kMediumN = 7168;
constexpr int kMediumCap = 16384;

struct MediumGroups {
    int total;
    const int *rep;          // [total]
    const uint64_t *key;     // [N] in raw order: id of group u = key[rep[u]]
};

__device__ __forceinline__ MediumGroups dedup_medium_body(const uint64_t *__restrict__ keys, int N,
                                                          int32_t *__restrict__ rep, int32_t *__restrict__ inverse,
                                                          int32_t *__restrict__ n_unique) {
    __shared__ uint64_t lkey[kMediumN];
    __shared__ int table[kMediumCap];        // raw index, later the group number, last the representatives
    __shared__ int wsum[kSmallThreads / 64 + 1];
    constexpr int kPer = kMediumN / kSmallThreads;
    const int per = (N + kSmallThreads - 1) / kSmallThreads;
    uint64_t key[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        key[i] = (i < per && n < N) ? keys[n] : 0;
    }
    for (int i = threadIdx.x; i < kMediumCap; i += kSmallThreads) table[i] = -1;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        if (i < per && n < N) lkey[n] = key[i];
    }
    __syncthreads();
    int slot[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        slot[i] = -1;
        if (i < per && n < N) {
            uint32_t h = mix64(key[i]) & (uint32_t)(kMediumCap - 1);
            // at most N <= kMediumCap / 2 slots are ever taken: a free one is always met
            for (int probe = 0; probe < kMediumCap; ++probe) {
                int cur = table[h];
                if (cur < 0) {
                    cur = atomicCAS(&table[h], -1, n);
                    if (cur < 0) { slot[i] = (int)h; break; }          // claimed
                }
                if (lkey[cur] == key[i]) {
                    atomicMin(&table[h], n);
                    slot[i] = (int)h;
                    break;
                }
                h = (h + 1) & (uint32_t)(kMediumCap - 1);
            }
        }
    }
    __syncthreads();

    int is_first[kPer];
    int mine = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        is_first[i] = (slot[i] >= 0 && table[slot[i]] == n) ? 1 : 0;
        mine += is_first[i];
    }
    int total;
    const int u0 = block_exclusive_scan(mine, wsum, total);   // barriers inside: all reads of the first indices done
    int u = u0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        if (is_first[i]) {
            rep[u] = threadIdx.x * per + i;
            table[slot[i]] = u;                                // the slot now carries its group number
            ++u;
        }
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int n = threadIdx.x * per + i;
        if (slot[i] >= 0) inverse[n] = table[slot[i]];
    }
    if (threadIdx.x == 0) *n_unique = total;
    __syncthreads();                                           // the group numbers are read: the table is free
    u = u0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        if (is_first[i]) table[u++] = threadIdx.x * per + i;   // representatives, for a consumer in this workgroup
    }
    return MediumGroups{total, table, lkey};
}

}  // namespace rnnlm
