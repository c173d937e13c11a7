// Grouping of identical 64-bit history ids on the device.
//
// The batched form of the cache lookup in Table 1 of the paper (steps 1-3 and 14): a
// history that was seen before is not computed again.  New histories are numbered in the
// order of first appearance (Table 1 step 10 numbers entries sequentially), which makes
// the result unique: rep[] ascending, inverse[] fixed.  Insertion order into the hash
// table is racy, so the order never comes from it: every slot keeps the MINIMUM raw
// index that hit it, a query is "first" iff it equals that minimum, and an exclusive
// prefix sum over the "first" flags gives the group numbers.
//
// Two implementations with identical results:
//   small  (N <= kSmallN): one workgroup, table and flags in LDS, one launch (N <= kMediumN: the
//          same with a table of raw indices and the keys in LDS once);
//   large  : table in the caller's workspace, five launches (the numbering is a grid-wide scan; six
//            beyond a million ids).
#include <mutex>

#include "dedup_small_body.h"
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

__host__ __device__ constexpr int table_capacity(int N) {
    int cap = 64;
    while (cap < 2 * N) cap <<= 1;
    return cap;
}

// ------------------------------------------------------------------------------ small path
__global__ __launch_bounds__(kSmallThreads) void dedup_small_kernel(
    const uint64_t *__restrict__ keys, int N, int32_t *__restrict__ rep,
    int32_t *__restrict__ inverse, int32_t *__restrict__ n_unique) {
    dedup_small_body(keys, N, rep, inverse, n_unique);
}

__global__ __launch_bounds__(kSmallThreads) void dedup_medium_kernel(
    const uint64_t *__restrict__ keys, int N, int32_t *__restrict__ rep,
    int32_t *__restrict__ inverse, int32_t *__restrict__ n_unique) {
    dedup_medium_body(keys, N, rep, inverse, n_unique);
}

// ------------------------------------------------------------------------------ large path
struct LargeWs {
    uint64_t *tkeys;   // [cap+1]
    int *tfirst;       // [cap+1]
    int *tgroup;       // [cap+1]
    int *slot;         // [N]
    int *block_total;  // [N / 1024 + 1]
};

__host__ inline LargeWs carve(void *ws, int N) {
    int cap = table_capacity(N);
    char *p = static_cast<char *>(ws);
    LargeWs w;
    w.tkeys = reinterpret_cast<uint64_t *>(p); p += (size_t)(cap + 2) * 8;
    w.tfirst = reinterpret_cast<int *>(p);     p += (size_t)(cap + 2) * 4;
    w.tgroup = reinterpret_cast<int *>(p);     p += (size_t)(cap + 2) * 4;
    w.slot = reinterpret_cast<int *>(p);       p += (size_t)N * 4;
    w.block_total = reinterpret_cast<int *>(p);
    return w;
}

__global__ void dedup_init_kernel(uint64_t *tkeys, int *tfirst, int cap) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= cap) {
        tkeys[i] = kEmpty;
        tfirst[i] = 0x7FFFFFFF;
    }
}

__global__ void dedup_insert_kernel(const uint64_t *__restrict__ keys, int N, uint64_t *tkeys,
                                    int *tfirst, int *slot, int cap) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    int s = find_or_insert(tkeys, cap, keys[n]);
    slot[n] = s;
    atomicMin(&tfirst[s], n);
}

// Group numbers in raw order = exclusive prefix sum over the "first" flags, so that every query is
// touched by a full grid: per-workgroup counts, then the numbering proper, which adds up the counts
// of the workgroups before it (beyond 1024 workgroups a scan of the counts by one workgroup comes in between).
constexpr int kRankThreads = 1024;

__device__ __forceinline__ int first_flag(int n, int N, const int *__restrict__ slot,
                                          const int *__restrict__ tfirst, int &s) {
    s = (n < N) ? slot[n] : 0;
    return (n < N && tfirst[s] == n) ? 1 : 0;
}

__global__ __launch_bounds__(kRankThreads) void dedup_count_kernel(int N, const int *__restrict__ slot,
                                                                   const int *__restrict__ tfirst,
                                                                   int *__restrict__ block_total) {
    __shared__ int wsum[kRankThreads / 64 + 1];
    int s, total;
    const int first = first_flag(blockIdx.x * kRankThreads + threadIdx.x, N, slot, tfirst, s);
    (void)block_exclusive_scan(first, wsum, total);
    if (threadIdx.x == 0) block_total[blockIdx.x] = total;
}

// In place: block_total[b] becomes the number of firsts before workgroup b; *n_unique the total.
__global__ __launch_bounds__(kRankThreads) void dedup_scan_kernel(int blocks, int *__restrict__ block_total,
                                                                  int32_t *__restrict__ n_unique) {
    __shared__ int wsum[kRankThreads / 64 + 1];
    int carry = 0;
    for (int base = 0; base < blocks; base += kRankThreads) {
        const int b = base + threadIdx.x;
        const int v = (b < blocks) ? block_total[b] : 0;
        int total;
        const int excl = carry + block_exclusive_scan(v, wsum, total);
        if (b < blocks) block_total[b] = excl;
        carry += total;
    }
    if (threadIdx.x == 0) *n_unique = carry;
}

// SCANNED: block_total holds the exclusive prefix already (dedup_scan_kernel ran).  Otherwise (at
// most kRankThreads workgroups) it holds the plain counts, every workgroup adds up the counts before
// its own, and the last one writes the total: one launch less.
template <bool SCANNED>
__global__ __launch_bounds__(kRankThreads) void dedup_number_kernel(int N, const int *__restrict__ slot,
                                                                    const int *__restrict__ tfirst,
                                                                    const int *__restrict__ block_total,
                                                                    int *__restrict__ tgroup,
                                                                    int32_t *__restrict__ rep,
                                                                    int32_t *__restrict__ n_unique) {
    __shared__ int wsum[kRankThreads / 64 + 1];
    const int n = blockIdx.x * kRankThreads + threadIdx.x;
    int s, total;
    const int first = first_flag(n, N, slot, tfirst, s);
    int before;
    if (SCANNED) {
        before = block_total[blockIdx.x];
    } else {
        const int v = ((int)threadIdx.x < (int)blockIdx.x) ? block_total[threadIdx.x] : 0;
        (void)block_exclusive_scan(v, wsum, before);
    }
    const int u = before + block_exclusive_scan(first, wsum, total);
    if (first) {
        rep[u] = n;
        tgroup[s] = u;
    }
    if (!SCANNED && blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) *n_unique = before + total;
}

__global__ void dedup_inverse_kernel(int N, const int *__restrict__ slot,
                                     const int *__restrict__ tgroup, int32_t *inverse) {
    int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n < N) inverse[n] = tgroup[slot[n]];
}

__global__ void dedup_empty_kernel(int32_t *n_unique) { *n_unique = 0; }

}  // namespace

namespace {
constexpr size_t workspace_bytes_for(int N) {
    if (N <= 0) return 0;
    const size_t bytes = (size_t)(table_capacity(N) + 2) * 16 + (size_t)N * 4 + ((size_t)N / kRankThreads + 2) * 4;
    return (bytes + 255) & ~(size_t)255;
}
}  // namespace

size_t dedup_workspace_bytes(int N) { return workspace_bytes_for(N); }

hipError_t launch_dedup(const uint64_t *keys, int N, int32_t *rep, int32_t *inverse,
                        int32_t *n_unique, void *workspace, hipStream_t stream) {
    if (N <= 0) {
        hipLaunchKernelGGL(dedup_empty_kernel, dim3(1), dim3(1), 0, stream, n_unique);
        return hipGetLastError();
    }
    if (N <= kSmallN) {
        hipLaunchKernelGGL(dedup_small_kernel, dim3(1), dim3(kSmallThreads), 0, stream, keys, N, rep,
                           inverse, n_unique);
        return hipGetLastError();
    }
    if (N <= kMediumN) {
        hipLaunchKernelGGL(dedup_medium_kernel, dim3(1), dim3(kSmallThreads), 0, stream, keys, N, rep,
                           inverse, n_unique);
        return hipGetLastError();
    }
    const int cap = table_capacity(N);
    LargeWs w = carve(workspace, N);
    hipLaunchKernelGGL(dedup_init_kernel, dim3((cap + 1 + 255) / 256), dim3(256), 0, stream, w.tkeys,
                       w.tfirst, cap);
    hipLaunchKernelGGL(dedup_insert_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, keys, N,
                       w.tkeys, w.tfirst, w.slot, cap);
    const int blocks = (N + kRankThreads - 1) / kRankThreads;
    hipLaunchKernelGGL(dedup_count_kernel, dim3(blocks), dim3(kRankThreads), 0, stream, N, w.slot, w.tfirst,
                       w.block_total);
    if (blocks <= kRankThreads) {
        hipLaunchKernelGGL(dedup_number_kernel<false>, dim3(blocks), dim3(kRankThreads), 0, stream, N, w.slot,
                           w.tfirst, w.block_total, w.tgroup, rep, n_unique);
    } else {
        hipLaunchKernelGGL(dedup_scan_kernel, dim3(1), dim3(kRankThreads), 0, stream, blocks, w.block_total,
                           n_unique);
        hipLaunchKernelGGL(dedup_number_kernel<true>, dim3(blocks), dim3(kRankThreads), 0, stream, N, w.slot,
                           w.tfirst, w.block_total, w.tgroup, rep, n_unique);
    }
    hipLaunchKernelGGL(dedup_inverse_kernel, dim3((N + 255) / 256), dim3(256), 0, stream, N, w.slot,
                       w.tgroup, inverse);
    return hipGetLastError();
}

}  // namespace rnnlm

// ---- grouping without a workspace argument, for callers that cannot allocate one -------------------
//
// The hash table, the slots and the counts of the large path live in a file-scope device array of a
// fixed size instead (2.3 MB: every GPU the library runs on holds its own copy until the process ends).
// In host code the array's name is only a stand-in for the symbol; the address the kernels take is
// asked for once per device with hipGetSymbolAddress and kept.
namespace {

constexpr size_t kStaticScratchBytes = rnnlm::workspace_bytes_for(RNNLM_DEDUP_STATIC_MAX_N);
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices];          // per device: where `scratch` lives there, or null before the first use

// Device address of `scratch` on the current device (looked up on first use, under a lock).
int static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return RNNLM_EDEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return RNNLM_EDEVICE;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return RNNLM_OK;
}

}  // namespace

namespace rnnlm {
// Called by rnnlm_load / rnnlm_hs_load as well, so that a caller who loads a model first never meets
// the look-up inside a stream capture.
int dedup_static_prepare() {
    void *p = nullptr;
    return static_scratch(&p);
}
}  // namespace rnnlm

extern "C" int rnnlm_dedup_static(const uint64_t *history_ids, int N, int32_t *rep, int32_t *inverse,
                                  int32_t *n_unique, void *hip_stream) {
    if (N < 0 || !n_unique) return RNNLM_EINVAL;
    if (N > 0 && (!history_ids || !rep || !inverse)) return RNNLM_EINVAL;
    if (N > RNNLM_DEDUP_STATIC_MAX_N) return RNNLM_ERANGE;
    void *ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc != RNNLM_OK) return rc;
    // the kernels clear what they use of the table themselves (a fill kernel, no memset node)
    hipError_t e = rnnlm::launch_dedup(history_ids, N, rep, inverse, n_unique, ws, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? RNNLM_OK : RNNLM_EDEVICE;
}
