// IndexTable and its inverse on the device (Section 3.2; Table 1 steps 5 and 7-12): a context
// -- the word it ends in and its hidden vector (Section 4.1) -- is stored once and stands for a
// 4-byte index from then on (Table 3), so that only indices have to travel.
//
// Inverse direction (context -> index), for N contexts given by value:
//   hash     a wave per eight contexts: 64-bit hash of the word and of every bit of the vector;
//   group    equal hashes of the call are grouped in order of first appearance (the grouping
//            kernel of the step);
//   lookup   the cache's lookup kernel on the hashes: found -> the stored index; new -> the next
//            indices in order of first appearance (Table 1 step 10), keys inserted;
//   commit   one wave per context: a new context is copied into the stores by its first
//            occurrence; every other one is compared word for word and bit for bit with the
//            context it was identified with (the stored one, or the first occurrence in this
//            call), so that a hash collision cannot go unnoticed: it is counted and the
//            context gets the index 0xFFFFFFFE instead of a wrong one.
// Forward direction (index -> context): a gather.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr uint32_t kNotStored = 0xFFFFFFFFu, kCollision = 0xFFFFFFFEu;

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)v, off, 64), hi = __shfl_xor((uint32_t)(v >> 32), off, 64);
        v += ((uint64_t)hi << 32) | lo;
    }
    return v;
}

// Rows of H floats can be walked in 16-byte pieces when H is a multiple of 4 and the buffer is
// 16-byte aligned (the stores of the table are).
__device__ __forceinline__ bool vec_rows(const void *p, int H) {
    return (H & 3) == 0 && (reinterpret_cast<uintptr_t>(p) & 15) == 0;
}

__device__ __forceinline__ void copy_row(uint32_t *dst, const uint32_t *src, int H, int lane, bool vec) {
    if (vec) {
        for (int j = 4 * lane; j < H; j += 256)
            *reinterpret_cast<u32x4 *>(dst + j) = *reinterpret_cast<const u32x4 *>(src + j);
    } else {
        for (int j = lane; j < H; j += 64) dst[j] = src[j];
    }
}

// The hash of a vector is multilinear: sum over the positions j of a_j * x_j (mod 2^64), x_j the bit
// pattern of element j and a_j an odd 64-bit multiplier derived from j -- order-free, so lanes and
// their partial sums combine freely, and two vectors that differ in one element never collide
// (a_j odd).  A wave hashes kHashRows consecutive contexts at once: the multipliers of its positions
// are computed once and the loads of all rows are in flight together.  The word is mixed in at
// the end.
constexpr int kHashRows = 8;

__device__ __forceinline__ uint64_t position_multiplier(int j) {
    return mix64_full((uint64_t)j + 0x632BE59BD9B4E019ull) | 1ull;
}

__global__ __launch_bounds__(256) void context_hash_kernel(const int32_t *__restrict__ word,
                                                            const float *__restrict__ h, int N, int H,
                                                            uint64_t *__restrict__ keys) {
    const int n0 = (blockIdx.x * 4 + (threadIdx.x >> 6)) * kHashRows, lane = threadIdx.x & 63;
    if (n0 >= N) return;
    const uint32_t *base = reinterpret_cast<const uint32_t *>(h);
    uint64_t acc[kHashRows];
#pragma unroll
    for (int r = 0; r < kHashRows; ++r) acc[r] = 0;
    if (vec_rows(h, H)) {                                // 16 bytes per lane and load
        for (int j = 4 * lane; j < H; j += 256) {
            uint64_t a[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = position_multiplier(j + i);
            u32x4 v[kHashRows];
#pragma unroll
            for (int r = 0; r < kHashRows; ++r)          // rows past N repeat the last one, unused
                v[r] = *reinterpret_cast<const u32x4 *>(base + (size_t)min(n0 + r, N - 1) * H + j);
#pragma unroll
            for (int r = 0; r < kHashRows; ++r)
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[r] += a[i] * (uint64_t)v[r][i];
        }
    } else {
        for (int j = lane; j < H; j += 64) {
            const uint64_t a = position_multiplier(j);
#pragma unroll
            for (int r = 0; r < kHashRows; ++r) acc[r] += a * (uint64_t)base[(size_t)min(n0 + r, N - 1) * H + j];
        }
    }
#pragma unroll
    for (int r = 0; r < kHashRows; ++r) {
        const uint64_t sum = wave_sum_u64(acc[r]);
        if (lane == 0 && n0 + r < N)
            keys[n0 + r] = mix64_full(sum ^ ((uint64_t)(uint32_t)word[n0 + r] * 0x9E3779B97F4A7C15ull));
    }
}

__global__ __launch_bounds__(256) void index_commit_kernel(IndexDev t, int N, const int32_t *__restrict__ word,
                                                            const float *__restrict__ h,
                                                            uint32_t *__restrict__ index) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    const int H = t.c.H;
    const int u = t.inverse[n];
    const int e = t.c.entry_of[u];
    const bool is_new = t.c.miss_of[u] >= 0;
    const int first = t.rep[u];
    const uint32_t *mine = reinterpret_cast<const uint32_t *>(h) + (size_t)n * H;
    const bool vec = vec_rows(h, H);
    bool differs = false;
    if (is_new && n == first) {
        if (e >= 0) {                                    // store the new context
            copy_row(reinterpret_cast<uint32_t *>(t.c.store_h) + (size_t)e * H, mine, H, lane, vec);
            if (lane == 0) t.store_word[e] = word[n];
        }
    } else {
        // `first` never equals n here when the reference is this call's first occurrence, and a
        // stored context is not written by this call: no read races a write
        const uint32_t *ref = is_new ? reinterpret_cast<const uint32_t *>(h) + (size_t)first * H
                                     : reinterpret_cast<const uint32_t *>(t.c.store_h) + (size_t)e * H;
        const int ref_word = is_new ? word[first] : t.store_word[e];
        bool d = word[n] != ref_word;
        if (vec) {
            for (int j = 4 * lane; j < H; j += 256) {
                const u32x4 a = *reinterpret_cast<const u32x4 *>(mine + j), b = *reinterpret_cast<const u32x4 *>(ref + j);
                d |= (a[0] != b[0]) | (a[1] != b[1]) | (a[2] != b[2]) | (a[3] != b[3]);
            }
        } else {
            for (int j = lane; j < H; j += 64) d |= mine[j] != ref[j];
        }
        differs = __any(d);
    }
    if (lane == 0) {
        if (differs) {
            atomicAdd(reinterpret_cast<unsigned long long *>(&t.errors[0]), 1ull);
            index[n] = kCollision;
        } else {
            index[n] = e >= 0 ? (uint32_t)e : kNotStored;
        }
    }
}

__global__ __launch_bounds__(256) void index_fetch_kernel(IndexDev t, int N, const uint32_t *__restrict__ index,
                                                           int32_t *__restrict__ word, float *__restrict__ h) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    const int H = t.c.H;
    const uint32_t i = index[n];
    float *dst = h + (size_t)n * H;
    if (i < (uint32_t)*t.c.n_entries) {
        copy_row(reinterpret_cast<uint32_t *>(dst), reinterpret_cast<const uint32_t *>(t.c.store_h) + (size_t)i * H, H,
                 lane, vec_rows(h, H));
        if (lane == 0) word[n] = t.store_word[i];
    } else {                                             // not an index this table holds
        for (int j = lane; j < H; j += 64) dst[j] = quiet_nan();
        if (lane == 0) {
            word[n] = -1;
            atomicAdd(reinterpret_cast<unsigned long long *>(&t.errors[1]), 1ull);
        }
    }
}

__global__ void index_clear_errors_kernel(IndexDev t) {
    if (threadIdx.x < 2) t.errors[threadIdx.x] = 0;
}

}  // namespace

hipError_t launch_index_reset(const IndexDev &t, hipStream_t stream) {
    hipError_t e = launch_cache_reset(t.c, stream);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(index_clear_errors_kernel, dim3(1), dim3(64), 0, stream, t);
    return hipGetLastError();
}

hipError_t launch_context_hash(const int32_t *word, const float *h, int N, int H, uint64_t *keys,
                               hipStream_t stream) {
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(context_hash_kernel, dim3((N + 4 * kHashRows - 1) / (4 * kHashRows)), dim3(256), 0, stream, word, h,
                       N, H, keys);
    return hipGetLastError();
}

hipError_t launch_index_commit(const IndexDev &t, int N, const int32_t *word, const float *h, uint32_t *index,
                               hipStream_t stream) {
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(index_commit_kernel, dim3((N + 3) / 4), dim3(256), 0, stream, t, N, word, h, index);
    return hipGetLastError();
}

hipError_t launch_index_fetch(const IndexDev &t, int N, const uint32_t *index, int32_t *word, float *h,
                              hipStream_t stream) {
    if (N <= 0) return hipSuccess;
    hipLaunchKernelGGL(index_fetch_kernel, dim3((N + 3) / 4), dim3(256), 0, stream, t, N, index, word, h);
    return hipGetLastError();
}

}  // namespace rnnlm
