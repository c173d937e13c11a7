// Output projection + log-sum-exp, LDS-tiled MFMA kernel for ANY hidden size, bf16 or fp32.
//
// Same result as the other output-projection kernels (normalising over all words of the
// vocabulary, Section 2.1 of the paper).  This is the form for models whose hidden block
// does not fit in registers (Hp > 512, e.g. the H = 1024 stress workload): both operands
// travel through LDS.
//   - a workgroup (4 waves, 2 x 2) owns 128 rows and walks the 128-word tiles of its
//     vocabulary split; a wave owns 64 words x 64 rows = four 32x32 accumulators;
//   - the reduction length is cut in chunks of 128 bytes per row (64 bf16 or 32 fp32); a chunk
//     is 128 rows of weights + 128 rows of hidden values (16 KB each), double-buffered, filled
//     by direct global->LDS loads;
//   - per 16-byte k-step a wave reads two A operands (words) and two B operands (rows) and
//     issues four MFMA 32x32x16 (bf16) or sixteen MFMA 32x32x2 (fp32, the full-precision
//     matrix instruction: one float per lane and operand, so a 16-byte read feeds four of
//     them; lane half g supplies k0 + 4 g + e to MFMA e, the same pairing for both operands);
//   - MFMA roles as in the staged kernel (A = words, B = rows): a lane holds sixteen logits
//     of ONE row per accumulator, the sum over words stays in the lane;
//   - after the last chunk of a tile the 64 logits per lane are exponentiated and added.
// LDS rows are 128 bytes (8 chunks of 16); chunk c of row r sits at c ^ ((r >> 1) & 7), which
// spreads the 16 lanes served together by one ds_read_b128 over all 16 bank groups.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kTThreads = 256;
constexpr int kTRows = 128, kTWords = 128;
constexpr int kTOperandBytes = 128 * 128;                     // 16 KB: one operand, one chunk of 128 B per row
constexpr int kTStageBytes = 2 * kTOperandBytes;              // words then rows
constexpr int kTLdsBytes = 2 * kTStageBytes + 2 * kTRows * 8; // + final cross-wave reduction
constexpr int kTLoads = 128 * 8 / kTThreads;                  // 16-byte loads per thread per operand (4)

// Four 32x32 accumulators += (two A operands) x (two B operands), 16 bytes of k per lane.
__device__ __forceinline__ void mma_2x2(f32x16 (&acc)[2][2], const bf16x8 (&a)[2], const bf16x8 (&d)[2]) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], d[j], acc[i][j], 0, 0, 0);
}
__device__ __forceinline__ void mma_2x2(f32x16 (&acc)[2][2], const f32x4 (&a)[2], const f32x4 (&d)[2]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], d[j][e], acc[i][j], 0, 0, 0);
}
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { typedef bf16x8 type; };
template <> struct Frag<float> { typedef f32x4 type; };

template <typename T, bool FIXED>
__global__ __launch_bounds__(kTThreads) void outproj_tiled_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev, int RG,
                                                                  int S) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int B = B_dev ? *B_dev : rows;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int rg = local % RG, split = xcd + kXcds * (local / RG);
    const int b0 = rg * kTRows;
    if (b0 >= B) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;                  // word half, row half of the tile
    const int Hp = m.Hp;
    constexpr int kTK = 128 / (int)sizeof(T);                  // k per chunk
    typedef typename Frag<T>::type frag_t;
    const T *Ot = static_cast<const T *>(m.Ot);
    const T *D = static_cast<const T *>(m.d);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int ntiles = m.Vp / kTWords;
    const int t_begin = (int)(((long long)split * ntiles) / S), t_end = (int)(((long long)(split + 1) * ntiles) / S);
    const int nk = Hp / kTK;                                   // chunks per tile
    const int nchunks = (t_end - t_begin) * nk;

    // loader: load q of this thread fills physical chunk f = q*256 + tid of an operand tile
    uint32_t voff[kTLoads];
#pragma unroll
    for (int q = 0; q < kTLoads; ++q) {
        const int f = q * kTThreads + tid;
        const int r = f >> 3, p = f & 7, c = p ^ ((r >> 1) & 7);
        voff[q] = (uint32_t)(r * Hp * (int)sizeof(T) + c * 16);
    }
    const uint32_t wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = lds_address(lds);
    auto issue = [&](int chunk, int stage) {
        const int t = t_begin + chunk / nk, k0 = (chunk % nk) * kTK;
        const T *wsrc = Ot + (size_t)t * kTWords * Hp + k0;
        const T *dsrc = D + (size_t)b0 * Hp + k0;
        const uint32_t base = lds0 + stage * kTStageBytes + wave_s * 1024;
#pragma unroll
        for (int q = 0; q < kTLoads; ++q) lds_dma_16(wsrc, voff[q], base + q * (kTThreads * 16));
#pragma unroll
        for (int q = 0; q < kTLoads; ++q)
            lds_dma_16(dsrc, voff[q], base + kTOperandBytes + q * (kTThreads * 16));
    };

    // LDS offsets of this lane's operands at k-step ks of a chunk: chunk index 2 ks + g of its row
    int aoff[2][4], boff[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int ra = wm * 64 + h * 32 + col, rb = wn * 64 + h * 32 + col;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            aoff[h][ks] = ra * 128 + (((2 * ks + g) ^ ((ra >> 1) & 7)) * 16);
            boff[h][ks] = kTOperandBytes + rb * 128 + (((2 * ks + g) ^ ((rb >> 1) & 7)) * 16);
        }
    }

    float mrun[2], srun[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) { mrun[h] = FIXED ? m.m2_fixed : -INFINITY; srun[h] = 0.f; }
    f32x16 acc[2][2];

    if (nchunks > 0) issue(0, 0);
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        const int stage = chunk & 1;
        wait_vmcnt<0>();                                       // my loads of this chunk have landed
        __syncthreads();                                       // everybody's; the other stage is free
        if (chunk + 1 < nchunks) issue(chunk + 1, stage ^ 1);
        const int kc = chunk % nk;
        if (kc == 0) {
#pragma unroll
            for (int a = 0; a < 2; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        }
        const char *st = lds + stage * kTStageBytes;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const frag_t a[2] = {*reinterpret_cast<const frag_t *>(st + aoff[0][ks]),
                                 *reinterpret_cast<const frag_t *>(st + aoff[1][ks])};
            const frag_t d[2] = {*reinterpret_cast<const frag_t *>(st + boff[0][ks]),
                                 *reinterpret_cast<const frag_t *>(st + boff[1][ks])};
            mma_2x2(acc, a, d);
        }
        if (kc == nk - 1) {                                    // the tile is complete: exp-and-add
            const int v0 = (t_begin + chunk / nk) * kTWords + wm * 64;
#pragma unroll
            for (int a = 0; a < 2; ++a) {
                f32x4 c[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) c[q] = *reinterpret_cast<const f32x4 *>(cvec + v0 + a * 32 + 8 * q + 4 * g);
#pragma unroll
                for (int b = 0; b < 2; ++b) {
                    float x[16];
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int i = 0; i < 4; ++i) x[4 * q + i] = fmaf(acc[a][b][4 * q + i], kLog2e, c[q][i]);
                    lse2_fold16<FIXED>(x, mrun[b], srun[b]);
                }
            }
        }
    }
    // lanes l and l+32 hold two halves of a row; waves wm = 0, 1 hold the two word halves
    float2 *red = reinterpret_cast<float2 *>(lds + 2 * kTStageBytes);      // [2 (wm)][128 rows]
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float m2 = __shfl_xor(mrun[h], 32, 64), s2 = __shfl_xor(srun[h], 32, 64);
        if (FIXED) srun[h] += s2;
        else lse2_merge(mrun[h], srun[h], m2, s2);
        if (g == 0) red[wm * kTRows + wn * 64 + h * 32 + col] = make_float2(mrun[h], srun[h]);
    }
    __syncthreads();
    if (tid < kTRows && b0 + tid < B) {
        float2 p = red[tid], q = red[kTRows + tid];
        if (FIXED) p.y += q.y;
        else lse2_merge(p.x, p.y, q.x, q.y);
        m.part[(size_t)(b0 + tid) * kMaxSplits + split] = p;
    }
}

template <typename T>
hipError_t launch_tiled_t(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, SplitInfo *splits,
                          hipStream_t stream) {
    static bool attr_set[2] = {false, false};
    const int which = fixed_offset ? 1 : 0;
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_tiled_kernel<T, true>)
                                  : reinterpret_cast<const void *>(outproj_tiled_kernel<T, false>);
    if (!attr_set[which]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kTLdsBytes);
        if (e != hipSuccess) return e;
        attr_set[which] = true;
    }
    const int RG = (rows + kTRows - 1) / kTRows, T128 = m.Vp / kTWords;
    // about two workgroups per compute unit (64 KB of LDS each) but never more splits than
    // 128-word tiles; splits in multiples of 8 so that the row groups streaming the same
    // weights share an XCD
    int Sx = 512 / (kXcds * RG);
    if (Sx > T128 / kXcds) Sx = T128 / kXcds;
    if (Sx < 1) Sx = 1;
    if (Sx > kMaxSplits / kXcds) Sx = kMaxSplits / kXcds;
    const int S = kXcds * Sx;
    splits->fixed_splits = S;
    splits->staged_wg_per_xcd = 0;
    dim3 grid(kXcds * RG * Sx), block(kTThreads);
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_tiled_kernel<T, true>), grid, block, kTLdsBytes, stream, m, rows, B_dev, RG, S);
    else
        hipLaunchKernelGGL((outproj_tiled_kernel<T, false>), grid, block, kTLdsBytes, stream, m, rows, B_dev, RG, S);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_outproj_tiled(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                SplitInfo *splits, hipStream_t stream) {
    if (m.dtype == RNNLM_BF16) return launch_tiled_t<bf16_t>(m, rows, B_dev, fixed_offset, splits, stream);
    return launch_tiled_t<float>(m, rows, B_dev, fixed_offset, splits, stream);
}

}  // namespace rnnlm
