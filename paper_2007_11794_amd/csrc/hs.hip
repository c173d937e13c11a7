// Hierarchical output layer (Section 2.1 of the paper): the words are the leaves of a Huffman
// tree, and the probability of a word is normalised only over the nodes on its path from the
// root: log p(w | h') = sum over the path nodes i of log sigmoid(+-theta_i . h'), + for code bit
// 0, - for code bit 1.  About log2 V dot products per queried word instead of V per row: the
// whole-vocabulary contraction of the full softmax disappears, what is left is a gather of node
// vectors (one contiguous row each), bound by L2 / HBM traffic.
//
// One wave per (query, word) pair, eight path nodes at a time: the eight node rows are requested
// together, the eight dot products are reduced over the wave at once, and the lane that ends up
// with node u turns its dot product into log sigmoid.  The tree comes with the model
// (rnnlm_hs_load); rnnlm_huffman_build below makes one from word frequencies on the host.
#include <algorithm>
#include <numeric>
#include <vector>

#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kHsBatch = 8;

// log sigmoid(x) = min(x, 0) - log(1 + exp(-|x|))
__device__ __forceinline__ float log_sigmoid_f32(float x) {
    const float t = fast_exp2(-fabsf(x) * kLog2e);
    return fminf(x, 0.f) - fast_log2(1.0f + t) * kLn2;
}

template <typename T>
__global__ __launch_bounds__(256) void hs_query_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int N, int K,
    const int32_t *__restrict__ query_word, const int32_t *__restrict__ row_of_query,
    const float *__restrict__ h_out, const float *__restrict__ base_score, float *__restrict__ logprob) {
    const int B = B_dev ? *B_dev : rows;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const long long pair = (long long)blockIdx.x * 4 + wave;
    if (pair >= (long long)N * K) return;                // wave-uniform; no barrier in this kernel
    const int n = (int)(pair / K);
    const int H = m.H, Hp = m.Hp;
    const int r_raw = row_of_query ? row_of_query[n] : n;
    const bool r_ok = r_raw >= 0 && r_raw < B;
    const int r = r_ok ? r_raw : 0;
    const int q_raw = query_word[pair];
    const bool q_ok = q_raw >= 0 && q_raw < m.V;
    const int q = q_ok ? q_raw : 0;
    const int off0 = m.path_off[q], len = m.path_off[q + 1] - off0;      // wave-uniform
    const T *Theta = static_cast<const T *>(m.Theta);
    const float *hrow = h_out + (size_t)r * H;
    const bool vec_ok = (H % 4) == 0;
    const int umine = batch_slot_of_lane(lane);
    float total = 0.f;
    for (int i0 = 0; i0 < len; i0 += kHsBatch) {
        const bool valid = i0 + umine < len;
        const uint32_t entry = valid ? (uint32_t)m.path_entry[off0 + i0 + umine] : 0u;
        const int node_mine = (int)(entry & 0x7FFFFFFFu);
        int node[kHsBatch];
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) node[u] = __builtin_amdgcn_readlane(node_mine, lane_of_batch_slot(u));
        float acc[kHsBatch];
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) acc[u] = 0.f;
        for (int j0 = lane * 8; j0 < Hp; j0 += 512) {
            float h8[8];
            load8_row(hrow, j0, H, vec_ok, 0.f, h8);
            float w8[kHsBatch][8];
#pragma unroll
            for (int u = 0; u < kHsBatch; ++u) load8_weights(Theta, (size_t)node[u] * Hp + j0, w8[u]);
#pragma unroll
            for (int u = 0; u < kHsBatch; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u] = fmaf(w8[u][i], h8[i], acc[u]);
        }
        const float x = wave_sum8(acc, lane);
        float term = valid ? log_sigmoid_f32((entry >> 31) ? -x : x) : 0.f;
        term += __shfl_xor(term, 32, 64);                // the eight slots differ in lane bits 5, 4, 3
        term += __shfl_xor(term, 16, 64);
        term += __shfl_xor(term, 8, 64);
        total += term;
    }
    if (lane == 0) {
        if (r_ok && q_ok) {
            logprob[pair] = base_score ? total - base_score[pair] : total;
        } else {
            atomicOr(m.flag, r_ok ? RNNLM_FLAG_BAD_QUERY_WORD : RNNLM_FLAG_BAD_ROW);
            logprob[pair] = quiet_nan();
        }
    }
}

// ---- the same for a raw query with several words: the paths of its K words share their upper
// nodes (every path starts at the root), so the workgroup of a raw query first collects the
// DISTINCT nodes of all K paths (a small LDS hash table, 23 KB in all: six workgroups per compute
// unit -- the kernel is a chain of dependent loads and lives on occupancy), computes one dot product per distinct
// node, and only then adds up log sigmoid along each path.  At the headline shape (K = 32, Zipf
// words) that is 163 instead of 304 node vectors per query.
// Two sizes of the workgroup of a raw query: up to 1024 path entries (all K words together) with 256
// threads, and up to 256 entries with 128 threads -- few words per query (a search step that extends
// every hypothesis by a handful of words): a third of the LDS, twice the queries in flight per
// compute unit, and the kernel lives on how many chains of dependent loads are in flight.
template <int THREADS, int LOG2_TABLE, int MAX_ENTRIES, int MAX_K>
struct HsShape {
    static constexpr int kThreads = THREADS;
    static constexpr int kLog2Table = LOG2_TABLE, kTable = 1 << LOG2_TABLE;   // slots of the node table (at most half full)
    static constexpr int kMaxEntries = MAX_ENTRIES;                          // path entries of one raw query
    static constexpr int kMaxK = MAX_K;
    static_assert(kTable >= 2 * MAX_ENTRIES && kTable <= 32768 && MAX_ENTRIES % THREADS == 0, "");
};
typedef HsShape<256, 11, 1024, 256> HsLarge;
typedef HsShape<128, 9, 256, 64> HsSmall;

// Dot products of the distinct nodes for a short hidden vector (Hp = 8 * LPR elements, LPR = 16 or
// 32): a node row takes only LPR lanes of a wave, so the wave works on 64 / LPR rows side by side,
// eight per lane group in flight: 32 (16) rows per wave and round trip to memory instead of 8.  Lane
// group g of wave w takes the nodes d = first + g + G * u, u = 0..7; the eight sums of a group are
// reduced together (a lane passes on the half it will not finish, as in wave_sum8).
template <typename T, int LPR, int THREADS>
__device__ __forceinline__ void hs_dots_short_rows(const T *Theta, const float *hrow, int H, int Hp, bool vec_ok,
                                                   const int *dnode, float *dx, int D, int wave, int lane) {
    static_assert(LPR == 16 || LPR == 32, "");
    constexpr int G = 64 / LPR, kPerWave = G * kHsBatch;
    const int g = lane / LPR, sl = lane % LPR, j0 = sl * 8;
    float h8[8];
    load8_row(hrow, j0, H, vec_ok, 0.f, h8);
    constexpr int top = LPR / 2;                           // 8 or 16
    const bool upa = (lane & top) != 0, upb = (lane & (top / 2)) != 0, upc = (lane & (top / 4)) != 0;
    const int u_mine = (upa ? 4 : 0) + (upb ? 2 : 0) + (upc ? 1 : 0);
    const bool writer = (lane & (top / 4 - 1)) == 0;
    auto fetch = [&](int first, float (&w8)[kHsBatch][8]) {
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) {
            const int d = first + g + G * u;
            const int node = d < D ? dnode[d] : 0;
            load8_weights(Theta, (size_t)node * Hp + j0, w8[u]);
        }
    };
    auto finish = [&](int first, const float (&w8)[kHsBatch][8]) {
        float acc[kHsBatch];
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) {
            acc[u] = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[u] = fmaf(w8[u][i], h8[i], acc[u]);
        }
        // three levels that halve the number of values a lane carries, then the rest of the butterfly
        float v4[4], v2[2];
#pragma unroll
        for (int i = 0; i < 4; ++i) v4[i] = (upa ? acc[4 + i] : acc[i]) + __shfl_xor(upa ? acc[i] : acc[4 + i], top, 64);
#pragma unroll
        for (int i = 0; i < 2; ++i) v2[i] = (upb ? v4[2 + i] : v4[i]) + __shfl_xor(upb ? v4[i] : v4[2 + i], top / 2, 64);
        float v = (upc ? v2[1] : v2[0]) + __shfl_xor(upc ? v2[0] : v2[1], top / 4, 64);
#pragma unroll
        for (int step = top / 8; step >= 1; step >>= 1) v += __shfl_xor(v, step, 64);
        const int d = first + g + G * u_mine;
        if (writer && d < D) dx[d] = v;
    };
    // two batches on their way at a time (the second may lie past the end: its loads fetch node 0)
    constexpr int stride = (THREADS / 64) * kPerWave;
    for (int first = wave * kPerWave; first < D; first += 2 * stride) {
        float wa[kHsBatch][8], wb[kHsBatch][8];
        fetch(first, wa);
        fetch(first + stride, wb);
        finish(first, wa);
        finish(first + stride, wb);
    }
}

// LPR: lanes per node row of the short-row form (16: Hp = 128, 32: Hp = 256), 0: any hidden size.
// Kernels of their own, so that the registers of the short-row form do not cost the general one occupancy.
template <typename T, int LPR, class S>
__global__ __launch_bounds__(S::kThreads) void hs_query_shared_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int N, int K,
    const int32_t *__restrict__ query_word, const int32_t *__restrict__ row_of_query,
    const float *__restrict__ h_out, const float *__restrict__ base_score, float *__restrict__ logprob) {
    __shared__ int wbase[S::kMaxK + 1];               // start of word k's entries
    __shared__ int woff[S::kMaxK];                    // where word k's path starts in the model's entries
    __shared__ uint16_t eslot[S::kMaxEntries];        // entry -> table slot of its node | code bit << 15
    __shared__ int tnode[S::kTable];                  // hash table: node (-1 free)
    __shared__ uint16_t tidx[S::kTable];              // slot -> index of its node among the distinct ones
    __shared__ int dnode[S::kMaxEntries];             // the distinct nodes
    __shared__ float dx[S::kMaxEntries];              // their dot products
    __shared__ int dcount;
    __shared__ int wsum[S::kThreads / 64 + 1];
    static_assert(S::kTable <= 32768, "slot index and code bit share sixteen bits");
    static_assert(S::kMaxK <= S::kThreads, "one word per thread in step 1");
    const int B = B_dev ? *B_dev : rows;
    const int n = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const int H = m.H, Hp = m.Hp;
    const int r_raw = row_of_query ? row_of_query[n] : n;
    const bool r_ok = r_raw >= 0 && r_raw < B;
    const int r = r_ok ? r_raw : 0;
    // 1. lengths of the K paths -> offsets (K <= 256: one word per thread)
    int len = 0;
    if (tid < K) {
        const int q_raw = query_word[(size_t)n * K + tid];
        const int q = (q_raw >= 0 && q_raw < m.V) ? q_raw : 0;
        const int o = m.path_off[q];
        len = m.path_off[q + 1] - o;
        woff[tid] = o;
    }
    for (int i = tid; i < S::kTable; i += S::kThreads) tnode[i] = -1;
    if (tid == 0) dcount = 0;
    int total;
    const int mybase = block_exclusive_scan(len, wsum, total);      // barriers inside
    if (tid < K) wbase[tid] = mybase;
    if (tid == 0) wbase[K] = total;
    __syncthreads();
    // 2. distinct nodes (a thread per path entry, all entries of a thread requested before the first
    //    is used: one round trip to memory for the whole query): the thread whose insertion claims
    //    a slot numbers the node; every entry remembers its slot and its code bit
    constexpr int kPerThread = S::kMaxEntries / S::kThreads;
    uint32_t entry[kPerThread];
#pragma unroll
    for (int c = 0; c < kPerThread; ++c) {
        const int e = tid + c * S::kThreads;
        entry[c] = 0u;
        if (e < total) {
            int lo = 0, hi = K;                                      // the word k with wbase[k] <= e < wbase[k + 1]
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (wbase[mid] <= e) lo = mid; else hi = mid;
            }
            entry[c] = (uint32_t)m.path_entry[woff[lo] + (e - wbase[lo])];
        }
    }
#pragma unroll
    for (int c = 0; c < kPerThread; ++c) {
        const int e = tid + c * S::kThreads;
        if (e < total) {
            const int node = (int)(entry[c] & 0x7FFFFFFFu);
            uint32_t h = (uint32_t)(node * 0x9E3779B1u) >> (32 - S::kLog2Table);
            for (int probe = 0; probe < S::kTable; ++probe) {
                const int old = atomicCAS(&tnode[h], -1, node);
                if (old == -1) {
                    const int d = atomicAdd(&dcount, 1);
                    dnode[d] = node;
                    tidx[h] = (uint16_t)d;
                    break;
                }
                if (old == node) break;
                h = (h + 1) & (S::kTable - 1);
            }
            eslot[e] = (uint16_t)(h | ((entry[c] >> 31) << 15));
        }
    }
    __syncthreads();
    const int D = dcount;
    // 3. one dot product per distinct node, eight nodes of a wave at a time
    const T *Theta = static_cast<const T *>(m.Theta);
    const float *hrow = h_out + (size_t)r * H;
    const bool vec_ok = (H % 4) == 0;
    const int umine = batch_slot_of_lane(lane);
    if constexpr (LPR != 0) hs_dots_short_rows<T, LPR, S::kThreads>(Theta, hrow, H, Hp, vec_ok, dnode, dx, D, wave, lane);
    else
    for (int d0 = wave * kHsBatch; d0 < D; d0 += (S::kThreads / 64) * kHsBatch) {
        const int node_mine = (d0 + umine < D) ? dnode[d0 + umine] : 0;
        int node[kHsBatch];
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) node[u] = __builtin_amdgcn_readlane(node_mine, lane_of_batch_slot(u));
        float acc[kHsBatch];
#pragma unroll
        for (int u = 0; u < kHsBatch; ++u) acc[u] = 0.f;
        for (int j0 = lane * 8; j0 < Hp; j0 += 512) {
            float h8[8];
            load8_row(hrow, j0, H, vec_ok, 0.f, h8);
            float w8[kHsBatch][8];
#pragma unroll
            for (int u = 0; u < kHsBatch; ++u) load8_weights(Theta, (size_t)node[u] * Hp + j0, w8[u]);
#pragma unroll
            for (int u = 0; u < kHsBatch; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u] = fmaf(w8[u][i], h8[i], acc[u]);
        }
        const float x = wave_sum8(acc, lane);
        if ((lane & 7) == 0 && d0 + umine < D) dx[d0 + umine] = x;
    }
    __syncthreads();
    // 4. log sigmoid of every path entry (a thread per entry; the terms go where the node table was,
    //    which nobody has probed since step 2), then eight lanes add up the terms of one word
    float *const eterm = reinterpret_cast<float *>(tnode);
    static_assert(S::kMaxEntries <= S::kTable, "the terms fit the node table");
#pragma unroll
    for (int c = 0; c < kPerThread; ++c) {
        const int e = tid + c * S::kThreads;
        if (e < total) {
            const uint32_t es = eslot[e];
            const float x = dx[tidx[es & 0x7FFFu]];
            eterm[e] = log_sigmoid_f32((es >> 15) ? -x : x);
        }
    }
    __syncthreads();
    for (int k = tid >> 3; k < K; k += S::kThreads / 8) {
        const int b0 = wbase[k], b1 = wbase[k + 1];
        float t = 0.f;
        for (int e = b0 + (tid & 7); e < b1; e += 8) t += eterm[e];
        t += __shfl_xor(t, 4, 64);
        t += __shfl_xor(t, 2, 64);
        t += __shfl_xor(t, 1, 64);
        if ((tid & 7) == 0) {
            const int qk = query_word[(size_t)n * K + k];
            const bool ok = qk >= 0 && qk < m.V;
            const size_t at = (size_t)n * K + k;
            if (r_ok && ok) {
                logprob[at] = base_score ? t - base_score[at] : t;
            } else {
                atomicOr(m.flag, r_ok ? RNNLM_FLAG_BAD_QUERY_WORD : RNNLM_FLAG_BAD_ROW);
                logprob[at] = quiet_nan();
            }
        }
    }
}

}  // namespace

hipError_t launch_hs_query(const ModelDev &m, int rows, const int *B_dev, int N, int K,
                           const int32_t *query_word, const int32_t *row_of_query, const float *h_out,
                           const float *base_score, float *logprob, hipStream_t stream) {
    if (N <= 0 || K <= 0) return hipSuccess;
    if (K >= 4 && K <= HsLarge::kMaxK && (long long)K * m.hs_max_len <= HsLarge::kMaxEntries) {
        // several words per query: one workgroup per raw query, shared path nodes computed once
        const bool small = K <= HsSmall::kMaxK && (long long)K * m.hs_max_len <= HsSmall::kMaxEntries;
        auto launch = [&](auto kernel, int threads) {
            hipLaunchKernelGGL(kernel, dim3(N), dim3(threads), 0, stream, m, rows, B_dev, N, K, query_word,
                               row_of_query, h_out, base_score, logprob);
        };
        auto pick = [&](auto tag) {
            using T = decltype(tag);
            if (small) {
                if (m.Hp == 128) launch(hs_query_shared_kernel<T, 16, HsSmall>, HsSmall::kThreads);
                else if (m.Hp == 256) launch(hs_query_shared_kernel<T, 32, HsSmall>, HsSmall::kThreads);
                else launch(hs_query_shared_kernel<T, 0, HsSmall>, HsSmall::kThreads);
            } else {
                if (m.Hp == 128) launch(hs_query_shared_kernel<T, 16, HsLarge>, HsLarge::kThreads);
                else if (m.Hp == 256) launch(hs_query_shared_kernel<T, 32, HsLarge>, HsLarge::kThreads);
                else launch(hs_query_shared_kernel<T, 0, HsLarge>, HsLarge::kThreads);
            }
        };
        if (m.dtype == RNNLM_BF16) pick(bf16_t{});
        else pick(float{});
        return hipGetLastError();
    }
    const long long pairs = (long long)N * K;
    const dim3 grid((unsigned)((pairs + 3) / 4));
    if (m.dtype == RNNLM_BF16)
        hipLaunchKernelGGL(hs_query_kernel<bf16_t>, grid, dim3(256), 0, stream, m, rows, B_dev, N, K, query_word,
                           row_of_query, h_out, base_score, logprob);
    else
        hipLaunchKernelGGL(hs_query_kernel<float>, grid, dim3(256), 0, stream, m, rows, B_dev, N, K, query_word,
                           row_of_query, h_out, base_score, logprob);
    return hipGetLastError();
}

}  // namespace rnnlm

// Huffman's method with two queues (host code): the words sorted by (frequency, id) ascending,
// and the inner nodes in order of creation, whose weights never decrease.  Every merge takes
// the two lightest queue heads, a word before an inner node of equal weight; the first taken is
// the child with code bit 0.  Inner nodes are numbered in order of creation, the root is V - 2.
extern "C" int rnnlm_huffman_build(int V, const double *frequency, int32_t *path_offset, int32_t *path_entry,
                                   size_t capacity, size_t *needed) {
    if (V < 2 || !frequency || !path_offset) return RNNLM_EINVAL;
    if (V > (1 << 30)) return RNNLM_ERANGE;
    for (int v = 0; v < V; ++v)
        if (!(frequency[v] >= 0.0)) return RNNLM_EINVAL;
    std::vector<int32_t> order, up;          // words by weight; parent of word v / of inner node V + i
    std::vector<double> weight;              // of the inner nodes
    std::vector<uint8_t> code;
    try {
        order.resize(V);
        up.assign(2 * (size_t)V - 1, -1);
        code.assign(2 * (size_t)V - 1, 0);
        weight.resize(V - 1);
    } catch (...) {
        return RNNLM_ENOMEM;
    }
    std::iota(order.begin(), order.end(), 0);
    std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
        return frequency[a] < frequency[b] || (frequency[a] == frequency[b] && a < b);
    });
    size_t next_word = 0, next_inner = 0;
    for (int created = 0; created < V - 1; ++created) {
        double sum = 0.0;
        for (int side = 0; side < 2; ++side) {
            const bool words_left = next_word < (size_t)V, inner_left = next_inner < (size_t)created;
            const bool take_word = words_left && (!inner_left || frequency[order[next_word]] <= weight[next_inner]);
            size_t child;
            if (take_word) {
                child = (size_t)order[next_word];
                sum += frequency[order[next_word++]];
            } else {
                child = (size_t)V + next_inner;
                sum += weight[next_inner++];
            }
            up[child] = V + created;
            code[child] = (uint8_t)side;
        }
        weight[created] = sum;
    }
    size_t total = 0;
    for (int v = 0; v < V; ++v) {
        size_t depth = 0;
        for (int32_t x = v; up[x] >= 0; x = up[x]) ++depth;
        path_offset[v] = (int32_t)total;
        if (path_entry && total + depth <= capacity) {
            size_t at = total + depth;
            for (int32_t x = v; up[x] >= 0; x = up[x])
                path_entry[--at] = (int32_t)((uint32_t)(up[x] - V) | ((uint32_t)code[x] << 31));
        }
        total += depth;
        if (total > 0x7FFFFFFFull) return RNNLM_ERANGE;
    }
    path_offset[V] = (int32_t)total;
    if (needed) *needed = total;
    return (path_entry && total <= capacity) ? RNNLM_OK : RNNLM_ERANGE;
}
