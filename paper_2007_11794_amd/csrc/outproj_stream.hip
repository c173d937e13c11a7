// Output projection + log-sum-exp for FEW rows: the weight-streaming kernels (bf16 models first,
// fp32 models at the end of the file).
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
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kThreads = kStreamThreads;
constexpr int kWaves = kStreamWaves;
constexpr int kRing = kStreamRing;
typedef StreamCursor Cursor;

template <int RB, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_stream_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev, int row0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // this launch serves rows row0 .. row0 + 32 RB - 1 (row0 a multiple of 32)
    const int B = (B_dev ? *B_dev : rows) - row0;
    if (B <= 0) return;                                       // uniform: no barrier is met
    outproj_stream_body<RB, FIXED>(m, B, row0, blockIdx.x, gridDim.x, lds);
}

// ------------------------------------------------------------------------------ fp32 models
// The same streaming for fp32 weights, at fp32 accuracy on the bf16 matrix cores: the weights come
// as fp32 in operand order (two 1 KB loads per operand of 32 words x 16 units) and are cut into
// their three bf16 terms in registers (x = x1 + x2 + x3, each term rounded to nearest); the hidden
// block is cut the same way while it is copied into LDS; six MFMAs per operand add the six
// largest of the nine cross terms (1.1, 1.2, 2.1, 1.3, 3.1, 2.2) in the fp32 accumulators.
constexpr int kGroup32 = 2;        // operands per group (four loads, as above)

// Two floats -> their three bf16 terms, packed pairwise (low half = a).
__device__ __forceinline__ void split3_pair(float a, float b, uint32_t &p1, uint32_t &p2, uint32_t &p3) {
    p1 = pack_bf16x2(a, b);
    const float ra = a - __uint_as_float(p1 << 16), rb = b - __uint_as_float(p1 & 0xFFFF0000u);
    p2 = pack_bf16x2(ra, rb);
    const float sa = ra - __uint_as_float(p2 << 16), sb = rb - __uint_as_float(p2 & 0xFFFF0000u);
    p3 = pack_bf16x2(sa, sb);
}
__device__ __forceinline__ void split3_x8(const f32x4 &lo, const f32x4 &hi, bf16x8 &t1, bf16x8 &t2, bf16x8 &t3) {
    uint32_t a[4], b[4], c[4];
    split3_pair(lo[0], lo[1], a[0], b[0], c[0]);
    split3_pair(lo[2], lo[3], a[1], b[1], c[1]);
    split3_pair(hi[0], hi[1], a[2], b[2], c[2]);
    split3_pair(hi[2], hi[3], a[3], b[3], c[3]);
    t1 = __builtin_bit_cast(bf16x8, u32x4{a[0], a[1], a[2], a[3]});
    t2 = __builtin_bit_cast(bf16x8, u32x4{b[0], b[1], b[2], b[3]});
    t3 = __builtin_bit_cast(bf16x8, u32x4{c[0], c[1], c[2], c[3]});
}

template <int RB, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_stream_f32_kernel(ModelDev m, int rows,
                                                                      const int *__restrict__ B_dev, int row0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int B = (B_dev ? *B_dev : rows) - row0;
    if (B <= 0) return;                                       // uniform: no barrier is met
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = m.Hp >> 4, GPB = KS / kGroup32;
    const int T = m.Vp / 32, S = gridDim.x, split = blockIdx.x;
    const int blk1 = (int)(((long long)(split + 1) * T) / S);
    const int blk0 = (int)(((long long)split * T) / S);
    const f32x4 *Of = static_cast<const f32x4 *>(m.Ofrag) + lane;           // [blk][ks][2][64] x 16 bytes
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    bf16x8 *dl = reinterpret_cast<bf16x8 *>(lds);                           // [3 terms][RB][KS][64]
    float2 *red = reinterpret_cast<float2 *>(lds + (size_t)3 * RB * KS * 1024);

    f32x4 ring[kRing][2 * kGroup32];
    Cursor in = {blk0 + wave, 0};
    auto issue = [&](f32x4(&dst)[2 * kGroup32]) {                          // always four loads (see above)
        const f32x4 *p = Of + (in.blk < blk1 ? ((size_t)in.blk * KS + in.part * kGroup32) * 128 : (size_t)0);
#pragma unroll
        for (int i = 0; i < 2 * kGroup32; ++i) dst[i] = p[i * 64];
        in.advance(GPB);
    };
#pragma unroll
    for (int st = 0; st < kRing - 1; ++st) issue(ring[st]);
    {   // hidden block: fp32 rows -> three bf16 terms in operand order (rows beyond B: stale scratch,
        // rows are independent and their results are dropped)
        const float *d = static_cast<const float *>(m.d) + (size_t)row0 * m.Hp;
        const int n = RB * KS * 64;
        for (int i = tid; i < n; i += kThreads) {
            const int l = i & 63, ks = (i >> 6) % KS, rb = (i >> 6) / KS;
            const float *src = d + (size_t)(32 * rb + (l & 31)) * m.Hp + 16 * ks + 8 * (l >> 5);
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(src), hi = *reinterpret_cast<const f32x4 *>(src + 4);
            bf16x8 t1, t2, t3;
            split3_x8(lo, hi, t1, t2, t3);
            dl[i] = t1;
            dl[n + i] = t2;
            dl[2 * n + i] = t3;
        }
    }
    __syncthreads();

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
    const int nd = RB * KS * 64;
    [&]() {
        for (;;) {
#pragma unroll
            for (int st = 0; st < kRing; ++st) {
                if (out.blk >= blk1) return;
                issue(ring[(st + kRing - 1) % kRing]);
#pragma unroll
                for (int i = 0; i < kGroup32; ++i) {
                    const int ks = out.part * kGroup32 + i;
                    bf16x8 w1, w2, w3;
                    split3_x8(ring[st][2 * i], ring[st][2 * i + 1], w1, w2, w3);
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        const int at = (rb * KS + ks) * 64 + lane;
                        const bf16x8 d1 = dl[at], d2 = dl[nd + at], d3 = dl[2 * nd + at];
                        // smallest terms first
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2, d2, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w3, d1, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, d3, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2, d1, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, d2, acc[rb], 0, 0, 0);
                        acc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w1, d1, acc[rb], 0, 0, 0);
                    }
                }
                if (out.part == GPB - 1) {                    // block complete: exp-and-add, next block
#pragma unroll
                    for (int rb = 0; rb < RB; ++rb) {
                        float x[16];
#pragma unroll
                        for (int q = 0; q < 4; ++q)
#pragma unroll
                            for (int i = 0; i < 4; ++i) x[4 * q + i] = fmaf(acc[rb][4 * q + i], kLog2e, cc[q][i]);
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
        if (tid < B) m.part[(size_t)(row0 + tid) * kMaxSplits + split] = make_float2(mm, ss);
    }
}

template <int RB>
hipError_t launch_rb(const ModelDev &m, int rows, const int *B_dev, int row0, bool fixed_offset, int S,
                     hipStream_t stream) {
    static size_t attr_bytes[4] = {0, 0, 0, 0};
    const bool f32 = m.dtype == RNNLM_F32;
    const int which = (fixed_offset ? 1 : 0) + (f32 ? 2 : 0);
    const size_t lds_bytes = stream_lds_bytes(f32 ? 3 : 1, RB, m.Hp >> 4);
    const void *fn = f32 ? (fixed_offset ? reinterpret_cast<const void *>(outproj_stream_f32_kernel<RB, true>)
                                         : reinterpret_cast<const void *>(outproj_stream_f32_kernel<RB, false>))
                         : (fixed_offset ? reinterpret_cast<const void *>(outproj_stream_kernel<RB, true>)
                                         : reinterpret_cast<const void *>(outproj_stream_kernel<RB, false>));
    if (attr_bytes[which] < lds_bytes) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return e;
        attr_bytes[which] = lds_bytes;
    }
    if (f32) {
        if (fixed_offset)
            hipLaunchKernelGGL((outproj_stream_f32_kernel<RB, true>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
        else
            hipLaunchKernelGGL((outproj_stream_f32_kernel<RB, false>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
    } else {
        if (fixed_offset)
            hipLaunchKernelGGL((outproj_stream_kernel<RB, true>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
        else
            hipLaunchKernelGGL((outproj_stream_kernel<RB, false>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
    }
    return hipGetLastError();
}

}  // namespace

// Rows the streaming kernel can take for this model: the hidden block (bf16 models: one copy;
// fp32 models: its three bf16 terms) must fit in LDS.
int outproj_stream_max_rows(const ModelDev &m) {
    if (!m.Ofrag || m.hs) return 0;
    if (m.dtype == RNNLM_BF16 && !m.dfrag) return 0;
    const int KS = m.Hp >> 4, terms = m.dtype == RNNLM_F32 ? 3 : 1;
    int rb = 0;
    for (int c = 1; c <= 4; c *= 2)
        if (stream_lds_bytes(terms, c, KS) <= 156 * 1024) rb = c;          // of the 160 KB a workgroup can have
    return 32 * rb;
}

// Rows beyond what one launch holds in LDS are served by further launches (each streams the weights
// again: worth it for a few passes only, the caller decides).
hipError_t launch_outproj_stream(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream) {
    const int per = outproj_stream_max_rows(m);
    if (per == 0) return hipErrorInvalidValue;
    const int T = m.Vp / 32;
    const int S = T < kMaxSplits ? T : kMaxSplits;
    *splits = fixed_split_info(S);
    for (int row0 = 0; row0 < rows; row0 += per) {
        const int n = rows - row0 < per ? rows - row0 : per;
        hipError_t e = n <= 32   ? launch_rb<1>(m, rows, B_dev, row0, fixed_offset, S, stream)
                       : n <= 64 ? launch_rb<2>(m, rows, B_dev, row0, fixed_offset, S, stream)
                                 : launch_rb<4>(m, rows, B_dev, row0, fixed_offset, S, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rnnlm
