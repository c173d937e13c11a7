// The weight-streaming output projection as device functions (bf16 models, then fp32 models): the
// kernels of its own (few rows known on the host) and the staged / three-term kernels (few rows
// known only on the device) run them.  See outproj_stream.hip for the design.
#pragma once

#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

constexpr int kStreamThreads = 512;
constexpr int kStreamWaves = kStreamThreads / 64;
constexpr int kStreamGroup = 4;          // MFMA operands (k-steps) per group of loads; Hp is a multiple of 64
constexpr int kStreamRing = 5;           // groups per wave: one being consumed, four in flight

struct StreamCursor {                    // walks the groups of the blocks blk, blk + kStreamWaves, ... of one wave
    int blk, part;
    __device__ __forceinline__ void advance(int groups_per_block) {
        if (++part == groups_per_block) { part = 0; blk += kStreamWaves; }
    }
};

// One launch's worth of streaming for the workgroup `split` of `S`: rows row0 .. row0 + 32 RB - 1 of
// the hidden block (B = number of valid ones among them, > 0), partials into m.part.  Needs
// stream_lds_bytes(1, RB, Hp / 16) bytes of LDS at `lds` and kStreamThreads threads; contains two
// workgroup barriers, so all threads of the workgroup must call it.
template <int RB, bool FIXED>
__device__ __forceinline__ void outproj_stream_body(const ModelDev &m, int B, int row0, int split, int S, char *lds) {
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = m.Hp >> 4, GPB = KS / kStreamGroup;
    const int T = m.Vp / 32;
    const int blk1 = part_begin(split + 1, T, S);
    const int blk0 = part_begin(split, T, S);
    const bf16x8 *Of = static_cast<const bf16x8 *>(m.Ofrag) + lane;
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    bf16x8 *dl = reinterpret_cast<bf16x8 *>(lds);
    float2 *red = reinterpret_cast<float2 *>(lds + (size_t)RB * KS * 1024);    // [kStreamWaves][RB * 32]

    // the hidden block first (its arrival is then not queued behind the weights)
    {
        const bf16x8 *src = static_cast<const bf16x8 *>(m.dfrag) + (size_t)(row0 >> 5) * KS * 64;
        const int n = RB * KS * 64;
        for (int i = tid; i < n; i += kStreamThreads) dl[i] = src[i];
    }
    bf16x8 ring[kStreamRing][kStreamGroup];
    StreamCursor in = {blk0 + wave, 0};
    // Always kStreamGroup loads, so that the number of younger loads behind any operand is the same on
    // every path and the waits for the ring stay partial; past the end of the wave's blocks the
    // loads go to the first kilobytes of the weights (cache hits, results unused).
    auto issue = [&](bf16x8(&dst)[kStreamGroup]) {
        const bf16x8 *p = Of + (in.blk < blk1 ? ((size_t)in.blk * KS + in.part * kStreamGroup) * 64 : (size_t)0);
#pragma unroll
        for (int i = 0; i < kStreamGroup; ++i) dst[i] = p[i * 64];
        in.advance(GPB);
    };
#pragma unroll
    for (int st = 0; st < kStreamRing - 1; ++st) issue(ring[st]);
    __syncthreads();                                          // hidden block visible to all waves

    StreamCursor out = {blk0 + wave, 0};
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
            for (int st = 0; st < kStreamRing; ++st) {
                if (out.blk >= blk1) return;
                issue(ring[(st + kStreamRing - 1) % kStreamRing]);
#pragma unroll
                for (int i = 0; i < kStreamGroup; ++i) {
                    const int ks = out.part * kStreamGroup + i;
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
        for (int w = 1; w < kStreamWaves; ++w) {
            const float2 p = red[w * (RB * 32) + tid];
            if (FIXED) ss += p.y;
            else lse2_merge(mm, ss, p.x, p.y);
        }
        if (tid < B) m.part[(size_t)(row0 + tid) * kMaxSplits + split] = make_float2(mm, ss);
    }
}

// ------------------------------------------------------------------------------ fp32 models
// The same streaming for fp32 weights, at fp32 accuracy on the bf16 matrix cores: the weights come
// as fp32 in operand order (two 1 KB loads per operand of 32 words x 16 units) and are cut into
// their three bf16 terms in registers (x = x1 + x2 + x3, each term rounded to nearest); the hidden
// block is cut the same way while it is copied into LDS; six MFMAs per operand add the six
// largest of the nine cross terms (1.1, 1.2, 2.1, 1.3, 3.1, 2.2) in the fp32 accumulators.
constexpr int kStreamGroup32 = 2;        // operands per group (four loads, as above)

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

// The fp32 form of outproj_stream_body: needs stream_lds_bytes(3, RB, Hp / 16) bytes of LDS.
template <int RB, bool FIXED>
__device__ __forceinline__ void outproj_stream_f32_body(const ModelDev &m, int B, int row0, int split, int S, char *lds) {
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int KS = m.Hp >> 4, GPB = KS / kStreamGroup32;
    const int T = m.Vp / 32;
    const int blk1 = part_begin(split + 1, T, S);
    const int blk0 = part_begin(split, T, S);
    const f32x4 *Of = static_cast<const f32x4 *>(m.Ofrag) + lane;           // [blk][ks][2][64] x 16 bytes
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    bf16x8 *dl = reinterpret_cast<bf16x8 *>(lds);                           // [3 terms][RB][KS][64]
    float2 *red = reinterpret_cast<float2 *>(lds + (size_t)3 * RB * KS * 1024);

    f32x4 ring[kStreamRing][2 * kStreamGroup32];
    StreamCursor in = {blk0 + wave, 0};
    auto issue = [&](f32x4(&dst)[2 * kStreamGroup32]) {                          // always four loads (see above)
        const f32x4 *p = Of + (in.blk < blk1 ? ((size_t)in.blk * KS + in.part * kStreamGroup32) * 128 : (size_t)0);
#pragma unroll
        for (int i = 0; i < 2 * kStreamGroup32; ++i) dst[i] = p[i * 64];
        in.advance(GPB);
    };
#pragma unroll
    for (int st = 0; st < kStreamRing - 1; ++st) issue(ring[st]);
    {   // hidden block: fp32 rows -> three bf16 terms in operand order (rows beyond B: stale scratch,
        // rows are independent and their results are dropped)
        const float *d = static_cast<const float *>(m.d) + (size_t)row0 * m.Hp;
        const int n = RB * KS * 64;
        for (int i = tid; i < n; i += kStreamThreads) {
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

    StreamCursor out = {blk0 + wave, 0};
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
            for (int st = 0; st < kStreamRing; ++st) {
                if (out.blk >= blk1) return;
                issue(ring[(st + kStreamRing - 1) % kStreamRing]);
#pragma unroll
                for (int i = 0; i < kStreamGroup32; ++i) {
                    const int ks = out.part * kStreamGroup32 + i;
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
        for (int w = 1; w < kStreamWaves; ++w) {
            const float2 p = red[w * (RB * 32) + tid];
            if (FIXED) ss += p.y;
            else lse2_merge(mm, ss, p.x, p.y);
        }
        if (tid < B) m.part[(size_t)(row0 + tid) * kMaxSplits + split] = make_float2(mm, ss);
    }
}

// terms = copies of the hidden block kept in LDS: 1 (bf16 models) or 3 (fp32 models)
__host__ __device__ inline size_t stream_lds_bytes(int terms, int RB, int KS) {
    return (size_t)terms * RB * KS * 1024 + (size_t)kStreamWaves * RB * 32 * sizeof(float2);
}

}  // namespace rnnlm
