// Output projection + log-sum-exp, LDS-staged bf16 MFMA kernel for Hp in {128, 256, 512}.
//
// What is computed is the same as in the plain kernel (normalising over all words of the
// vocabulary, Section 2.1 of the paper); this is the fast form for batches of >= 128 rows.
//
// Shape of the work.  The hidden block d = h' - 1/2 is tiny (rows x Hp bf16, 1 MB at
// 1024 x 512) and the output weights Ot[Vp][Hp] are large (64 MB at V = 65536), so the
// weights are streamed exactly once per row group and the hidden block never moves:
//   - a workgroup (8 waves) owns 256 rows; each wave keeps ITS 32 rows of d for the whole
//     reduction length in registers (Hp/16 MFMA B-operands, 128 VGPRs at Hp = 512);
//   - the weights of 64 words (64 x Hp bf16, 64 KB at Hp = 512) form one LDS stage, filled
//     by direct global->LDS loads (no VGPR round trip) one tile ahead of use; two stages;
//   - per tile a wave issues 2 x Hp/16 MFMA 32x32x16: A = 32 words x 16 k from LDS,
//     B = 16 k x 32 rows from registers, so lane l holds 16 logits of ONE row and the sum
//     over words stays inside the lane;
//   - the exp-and-add of tile t is interleaved, instruction by instruction, with the MFMAs
//     of tile t+1, so the vector ALU works in the shadow of the matrix core.
// LDS rows are XOR-swizzled in 16-byte chunks (chunk c of word r sits at c ^ (r & 15)) so
// that the 16 lanes served together by one ds_read_b128 hit 16 different bank groups.  The
// direct loads write LDS linearly (lane i -> base + 16 i), so the swizzle is applied on the
// global side: lane i fetches the chunk that belongs at position i.
//
// Work split (staged_plan): workgroup id modulo 8 is the XCD; vocabulary split s runs on
// XCD s % 8, with all row groups of that split next to each other, so the row groups that
// stream the same weights hit in the same 4 MB L2 and HBM is read once.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

typedef __attribute__((address_space(3))) void *lds_ptr_t;

__device__ __forceinline__ lds_ptr_t to_lds(const void *p) {
    return reinterpret_cast<lds_ptr_t>(reinterpret_cast<uintptr_t>(p));
}

constexpr int kThreads = 512;
constexpr int kCvecBytes = kStagedWords * 4;

template <int HP>
struct StagedCfg {
    static constexpr int KS = HP / 16;                       // MFMA k-steps
    static constexpr int CPR = HP / 8;                       // 16-byte chunks per word row
    static constexpr int kStageChunks = kStagedWords * CPR;
    static constexpr int kStageBytes = kStageChunks * 16;
    static constexpr int kLoadsPerThread = kStageChunks / kThreads;
    static constexpr int kLdsBytes = 2 * kStageBytes + 2 * kCvecBytes;
    static_assert(kStageChunks % kThreads == 0, "stage must be a whole number of loads per thread");
    static_assert(CPR >= 16, "swizzle needs at least 16 chunks per row");
};

// Start the direct global->LDS loads of one 64-word tile (weights and constants).
template <int HP>
__device__ __forceinline__ void issue_tile_loads(const bf16_t *__restrict__ Ot,
                                                 const float *__restrict__ cvec, int v0, char *stage,
                                                 char *cstage) {
    using C = StagedCfg<HP>;
    const int tid = threadIdx.x, wave = tid >> 6;
#pragma unroll
    for (int q = 0; q < C::kLoadsPerThread; ++q) {
        const int f = q * kThreads + tid;                    // physical chunk this lane fills
        const int r = f / C::CPR, p = f % C::CPR;
        const int c = p ^ (r & 15);                          // logical chunk that belongs there
        const bf16_t *src = Ot + (size_t)(v0 + r) * HP + c * 8;
        char *dst_wave = stage + (size_t)(q * kThreads + wave * 64) * 16;   // wave-uniform base
        __builtin_amdgcn_global_load_lds(src, to_lds(dst_wave), 16, 0, 0);
    }
    if (tid < kStagedWords / 4)
        __builtin_amdgcn_global_load_lds(cvec + v0 + tid * 4, to_lds(cstage), 16, 0, 0);
}

template <int HP, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_staged_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev,
                                                                  int wg_per_xcd) {
    using C = StagedCfg<HP>;
    constexpr int KS = C::KS;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int B = B_dev ? *B_dev : rows;
    const StagedPlan plan = staged_plan(B, wg_per_xcd);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const bf16_t *Ot = static_cast<const bf16_t *>(m.Ot);
    const float *cvec = FIXED ? m.cvec_fixed : m.cvec;
    const int T = m.Vp / kStagedWords;
    const int items = plan.RG * plan.Sx;
    const int swz = col & 15;

    for (int item = local; item < items; item += wg_per_xcd) {
        const int rg = item % plan.RG, split = xcd + kXcds * (item / plan.RG);
        const int t_begin = (int)(((long long)split * T) / plan.S);
        const int t_end = (int)(((long long)(split + 1) * T) / plan.S);
        const int b = rg * kStagedRows + wave * 32 + col;     // this lane's row

        // this wave's rows of d, all k, as MFMA B-operands (rows beyond B hold stale finite or
        // NaN scratch; rows are independent and those lanes' results are dropped)
        bf16x8 dreg[KS];
        {
            const bf16_t *drow = static_cast<const bf16_t *>(m.d) + (size_t)b * HP + 8 * g;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) dreg[ks] = *reinterpret_cast<const bf16x8 *>(drow + 16 * ks);
        }

        float mrun = FIXED ? m.m2_fixed : -INFINITY, srun = 0.f;
        // logits of the previous tile, still to be exponentiated; -inf adds 2^-inf = 0
        f32x16 pacc0, pacc1;
#pragma unroll
        for (int i = 0; i < 16; ++i) { pacc0[i] = -INFINITY; pacc1[i] = -INFINITY; }

        if (t_begin < t_end)
            issue_tile_loads<HP>(Ot, cvec, t_begin * kStagedWords, lds, lds + 2 * C::kStageBytes);

        for (int t = t_begin; t < t_end; ++t) {
            const int sidx = (t - t_begin) & 1;
            char *stage = lds + sidx * C::kStageBytes;
            const char *cstage = lds + 2 * C::kStageBytes + sidx * kCvecBytes;
            __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): my loads of tile t landed
            __syncthreads();                                  // everyone's landed; stage sidx^1 is free
            if (t + 1 < t_end)
                issue_tile_loads<HP>(Ot, cvec, (t + 1) * kStagedWords, lds + (sidx ^ 1) * C::kStageBytes,
                                     lds + 2 * C::kStageBytes + (sidx ^ 1) * kCvecBytes);

            // accumulators start from the per-word constants
            f32x16 acc0, acc1;
            {
                const f32x4 *cn = reinterpret_cast<const f32x4 *>(cstage);
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 c0 = cn[2 * q + g], c1 = cn[8 + 2 * q + g];
#pragma unroll
                    for (int i = 0; i < 4; ++i) { acc0[4 * q + i] = c0[i]; acc1[4 * q + i] = c1[i]; }
                }
            }
            const char *row0 = stage + (size_t)col * (C::CPR * 16);
            const char *row1 = row0 + (size_t)32 * (C::CPR * 16);

            if (FIXED) {
                // one slice of the previous tile's exp-and-add per k-step
                constexpr int EPS = 32 / KS > 0 ? 32 / KS : 1;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int p = ((2 * ks + g) ^ swz) * 16;
                    bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(row0 + p);
                    bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(row1 + p);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, dreg[ks], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, dreg[ks], acc1, 0, 0, 0);
#pragma unroll
                    for (int e = ks * EPS; e < (ks + 1) * EPS && e < 32; ++e) {
                        float z = e < 16 ? pacc0[e & 15] : pacc1[e & 15];
                        srun += fast_exp2(z * kLog2e);
                    }
                }
            } else {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const int p = ((2 * ks + g) ^ swz) * 16;
                    bf16x8 a0 = *reinterpret_cast<const bf16x8 *>(row0 + p);
                    bf16x8 a1 = *reinterpret_cast<const bf16x8 *>(row1 + p);
                    acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, dreg[ks], acc0, 0, 0, 0);
                    acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, dreg[ks], acc1, 0, 0, 0);
                    if (ks == KS / 4 || ks == (3 * KS) / 4) {
                        const f32x16 &pa = (ks == KS / 4) ? pacc0 : pacc1;
                        float mx = pa[0];
#pragma unroll
                        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, pa[i]);
                        mx *= kLog2e;
                        const float mn = fmaxf(mrun, mx);
                        if (mn != -INFINITY) {
                            float tsum = 0.f;
#pragma unroll
                            for (int i = 0; i < 16; ++i) tsum += fast_exp2(fmaf(pa[i], kLog2e, -mn));
                            srun = srun * fast_exp2(mrun - mn) + tsum;
                            mrun = mn;
                        }
                    }
                }
            }
            pacc0 = acc0;
            pacc1 = acc1;
        }

        {                                                     // the last tile's exp-and-add
            if (FIXED) {
#pragma unroll
                for (int i = 0; i < 16; ++i) srun += fast_exp2(pacc0[i] * kLog2e);
#pragma unroll
                for (int i = 0; i < 16; ++i) srun += fast_exp2(pacc1[i] * kLog2e);
            } else {
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const f32x16 &pa = h ? pacc1 : pacc0;
                    float mx = pa[0];
#pragma unroll
                    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, pa[i]);
                    mx *= kLog2e;
                    const float mn = fmaxf(mrun, mx);
                    if (mn != -INFINITY) {
                        float tsum = 0.f;
#pragma unroll
                        for (int i = 0; i < 16; ++i) tsum += fast_exp2(fmaf(pa[i], kLog2e, -mn));
                        srun = srun * fast_exp2(mrun - mn) + tsum;
                        mrun = mn;
                    }
                }
            }
        }
        // lanes l and l+32 hold the two halves of a row
        const float m2 = __shfl_xor(mrun, 32, 64), s2 = __shfl_xor(srun, 32, 64);
        if (FIXED) srun += s2;
        else lse2_merge(mrun, srun, m2, s2);
        if (g == 0 && b < B) m.part[(size_t)b * kMaxSplits + split] = make_float2(mrun, srun);
        __syncthreads();                                      // LDS is reused by the next item
    }
}

template <int HP>
hipError_t launch_hp(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, int wg_per_xcd,
                     hipStream_t stream) {
    using C = StagedCfg<HP>;
    static bool attr_set[2] = {false, false};
    const int which = fixed_offset ? 1 : 0;
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_staged_kernel<HP, true>)
                                  : reinterpret_cast<const void *>(outproj_staged_kernel<HP, false>);
    if (!attr_set[which]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set[which] = true;
    }
    dim3 grid(kXcds * wg_per_xcd), block(kThreads);
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_staged_kernel<HP, true>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd);
    else
        hipLaunchKernelGGL((outproj_staged_kernel<HP, false>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd);
    return hipGetLastError();
}

}  // namespace

bool outproj_staged_supported(const ModelDev &m) {
    return m.dtype == RNNLM_BF16 && (m.Hp == 128 || m.Hp == 256 || m.Hp == 512);
}

hipError_t launch_outproj_staged(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream) {
    // One workgroup per compute unit: 256 CUs in 8 XCDs.
    const int wg_per_xcd = 32;
    splits->fixed_splits = 0;
    splits->staged_wg_per_xcd = wg_per_xcd;
    switch (m.Hp) {
        case 128: return launch_hp<128>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        case 256: return launch_hp<256>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        case 512: return launch_hp<512>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace rnnlm
