// Output projection + log-sum-exp for FEW rows (bf16 models): the weight-streaming kernel.
//
// What is computed is the same as in the other output-projection kernels (normalising over
// all words of the vocabulary, Section 2.1 of the paper).  With a handful of distinct
// histories in a step -- the paper's search re-asks the same context most of the time
// (Section 5.2), so few rows are left after the lookup -- the contraction is a thin one:
// every weight is used for at most a few dozen rows, and the time is the time to read the
// output weights once.  So this kernel is built around the memory system, not the matrix core:
//   - the weights are read from a second copy kept in MFMA-operand order (Ofrag: one operand
//     of a wave = 32 words x 16 units = 1 KB contiguous), so every load instruction of a wave
//     is one fully coalesced kilobyte straight into the registers the MFMA reads: no LDS
//     round trip, no barrier, no partial cache lines;
//   - a wave owns whole 32-word blocks and keeps a ring of kRing groups of kGroup operands in
//     flight (16 KB per wave, 128 KB per CU with 8 waves, 32 MB over the chip: more than
//     bandwidth x latency of HBM), waves never synchronise inside the loop;
//   - the hidden block (<= 32 RB rows, times log2 e, already in operand order) sits in LDS and is
//     read per MFMA; one weight operand feeds RB MFMAs;
//   - exp-and-add per block in registers as elsewhere; at the end the eight waves' (max, sum)
//     pairs are merged through LDS in a fixed order: one partial per row and workgroup.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kGroup = 4;          // MFMA operands (k-steps) per group of loads; Hp is a multiple of 64
constexpr int kRing = 5;           // groups per wave: one being consumed, four in flight

struct Cursor {                    // walks the groups of the blocks blk, blk + kWaves, ... of one wave
    int blk, part;
    __device__ __forceinline__ void advance(int groups_per_block) {
        if (++part == groups_per_block) { part = 0; blk += kWaves; }
    }
};

template <int RB, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_stream_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int B = B_dev ? *B_dev : rows;
    if (B <= 0) return;                                       // uniform: no barrier is met
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = m.Hp >> 4, GPB = KS / kGroup;
    const int T = m.Vp / 32, S = gridDim.x, split = blockIdx.x;
    const int blk1 = (int)(((long long)(split + 1) * T) / S);
    const int blk0 = (int)(((long long)split * T) / S);
    const bf16x8 *Of = static_cast<const bf16x8 *>(m.Ofrag) + lane;
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    bf16x8 *dl = reinterpret_cast<bf16x8 *>(lds);
    float2 *red = reinterpret_cast<float2 *>(lds + (size_t)RB * KS * 1024);    // [kWaves][RB * 32]

    // the hidden block first (its arrival is then not queued behind the weights)
    {
        const bf16x8 *src = static_cast<const bf16x8 *>(m.dfrag);
        const int n = RB * KS * 64;
        for (int i = tid; i < n; i += kThreads) dl[i] = src[i];
    }
    bf16x8 ring[kRing][kGroup];
    Cursor in = {blk0 + wave, 0};
    // Always kGroup loads, so that the number of younger loads behind any operand is the same on
    // every path and the waits for the ring stay partial; past the end of the wave's blocks the
    // loads go to the first kilobytes of the weights (cache hits, results unused).
    auto issue = [&](bf16x8(&dst)[kGroup]) {
        const bf16x8 *p = Of + (in.blk < blk1 ? ((size_t)in.blk * KS + in.part * kGroup) * 64 : (size_t)0);
#pragma unroll
        for (int i = 0; i < kGroup; ++i) dst[i] = p[i * 64];
        in.advance(GPB);
    };
#pragma unroll
    for (int st = 0; st < kRing - 1; ++st) issue(ring[st]);
    __syncthreads();                                          // hidden block visible to all waves

    Cursor out = {blk0 + wave, 0};
    f32x16 acc[RB];
    float mrun[RB], srun[RB];
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        mrun[rb] = FIXED ? m.m2_fixed : -INFINITY;
        srun[rb] = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
    }
    f32x4 cc[4];
    auto load_constants = [&]() {
        const int blk = out.blk < blk1 ? out.blk : blk0;
#pragma unroll
        for (int q = 0; q < 4; ++q) cc[q] = *reinterpret_cast<const f32x4 *>(cvec + blk * 32 + 8 * q + 4 * g);
    };
    load_constants();
    // The wave leaves the unrolled ring loop from wherever its last group falls (a return out of
    // the lambda, never a skip that rejoins the loop: the compiler sizes each wait by the path
    // with the fewest younger loads).
    [&]() {
        for (;;) {
#pragma unroll
            for (int st = 0; st < kRing; ++st) {
                if (out.blk >= blk1) return;
                issue(ring[(st + kRing - 1) % kRing]);
#pragma unroll
                for (int i = 0; i < kGroup; ++i) {
                    const int ks = out.part * kGroup + i;
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb)
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[st][i], dl[(rb * KS + ks) * 64 + lane],
                                                                          acc[rb], 0, 0, 0);
                }
                if (out.part == GPB - 1) {                    // block complete: exp-and-add, next block
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        float x[16];
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[4 * q + i] = acc[rb][4 * q + i] + cc[q][i];
                        lse2_fold16<FIXED>(x, mrun[rb], srun[rb]);
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[rb][i] = 0.f;
                    }
                    out.advance(GPB);
                    load_constants();
                } else {
                    out.advance(GPB);
                }
            }
        }
    }();
    // lanes l and l + 32 hold the two halves of a row; then the eight waves of the workgroup
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        const float m2 = __shfl_xor(mrun[rb], 32, 64), s2 = __shfl_xor(srun[rb], 32, 64);
        if (FIXED) srun[rb] += s2;
        else lse2_merge(mrun[rb], srun[rb], m2, s2);
        if (g == 0) red[wave * (RB * 32) + rb * 32 + col] = make_float2(mrun[rb], srun[rb]);
    }
    __syncthreads();
    if (tid < RB * 32) {
        float mm = red[tid].x, ss = red[tid].y;
        for (int w = 1; w < kWaves; ++w) {
            const float2 p = red[w * (RB * 32) + tid];
            if (FIXED) ss += p.y;
            else lse2_merge(mm, ss, p.x, p.y);
        }
        if (tid < B) m.part[(size_t)tid * kMaxSplits + split] = make_float2(mm, ss);
    }
}

size_t stream_lds_bytes(int RB, int KS) { return (size_t)RB * KS * 1024 + (size_t)kWaves * RB * 32 * sizeof(float2); }

template <int RB>
hipError_t launch_rb(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, int S, hipStream_t stream) {
    static size_t attr_bytes[2] = {0, 0};
    const int which = fixed_offset ? 1 : 0;
    const size_t lds_bytes = stream_lds_bytes(RB, m.Hp >> 4);
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_stream_kernel<RB, true>)
                                  : reinterpret_cast<const void *>(outproj_stream_kernel<RB, false>);
    if (attr_bytes[which] < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_bytes[which] = lds_bytes;
    }
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_stream_kernel<RB, true>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev);
    else
        hipLaunchKernelGGL((outproj_stream_kernel<RB, false>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev);
    return hipGetLastError();
}

}  // namespace

// Rows the streaming kernel can take for this model: the hidden block must fit in LDS.
int outproj_stream_max_rows(const ModelDev &m) {
    if (m.dtype != RNNLM_BF16 || !m.Ofrag || !m.dfrag) return 0;
    const int KS = m.Hp >> 4;
    int rb = 0;
    for (int c = 1; c <= 4; c *= 2)
        if (stream_lds_bytes(c, KS) <= 144 * 1024) rb = c;
    return 32 * rb;
}

hipError_t launch_outproj_stream(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream) {
    if (rows > outproj_stream_max_rows(m)) return hipErrorInvalidValue;
    const int T = m.Vp / 32;
    const int S = T < kMaxSplits ? T : kMaxSplits;
    splits->fixed_splits = S;
    splits->staged_wg_per_xcd = 0;
    if (rows <= 32) return launch_rb<1>(m, rows, B_dev, fixed_offset, S, stream);
    if (rows <= 64) return launch_rb<2>(m, rows, B_dev, fixed_offset, S, stream);
    return launch_rb<4>(m, rows, B_dev, fixed_offset, S, stream);
}

}  // namespace rnnlm
