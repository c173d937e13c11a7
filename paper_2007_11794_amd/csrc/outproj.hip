// Output projection fused with the log-sum-exp over the vocabulary:
//     z[b][v] = bias[v] + sum_j O[j][v] h'[b][j],      lse[b] = log sum_v exp z[b][v]
// (normalising over all words of the vocabulary is the cost Section 2.1 of the paper
// names).  The B x V logits exist only in registers; what reaches memory is, per row and
// per vocabulary split, one (max, sum) pair of the base-2 log-sum-exp.
//
// With h' = 1/2 + d the logit is  z = (bias + 1/2 colsum(O)) + sum_j O[j][v] d[j]; the
// bracket, times log2(e), is the per-word constant cvec2[v] (-inf for the padded words
// beyond V, which then add 2^-inf = 0).  Two ways to take the sum:
//   running maximum  per lane (m, s): always valid;
//   fixed offset     since |d| <= 1/2 every base-2 logit is <= m2_fixed, a bound computed
//                    at load time; s = sum 2^(x - m2_fixed) needs no maximum and no
//                    rescaling.  Used when the bound is tight enough for fp32.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

// Accumulate sixteen base-2 logits of one row into (m, s).
template <bool FIXED>
__device__ __forceinline__ void lse2_accumulate16(const float (&x)[16], float &m, float &s) {
    if (FIXED) {
#pragma unroll
        for (int i = 0; i < 16; ++i) s += fast_exp2(x[i]);       // x already has the offset removed
    } else {
        float mx = x[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) mx = fmaxf(mx, x[i]);
        float mn = fmaxf(m, mx);
        if (mn != -INFINITY) {
            float t = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) t += fast_exp2(x[i] - mn);
            s = s * fast_exp2(m - mn) + t;
            m = mn;
        }
    }
}

// ------------------------------------------------------------------- plain bf16 MFMA kernel
// Any Hp (multiple of 16), any Vp (multiple of 32).  One wave owns 32 rows and walks the
// 32-word blocks of its vocabulary split; operands come straight from global memory (L1/L2).
// MFMA roles: A = 32 words x 16 k of Ot, B = 16 k x 32 rows of d, so that lane l holds
// sixteen logits of ONE row (l % 32) and the sum over words needs no cross-lane traffic
// until the very end (lanes l and l + 32 share a row).
template <bool FIXED>
__global__ __launch_bounds__(256) void outproj_plain_bf16_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int blocks_per_split, int splits) {
    const int B = B_dev ? *B_dev : rows;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, g = lane >> 5;
    const int b0 = (blockIdx.y * 4 + wave) * 32;
    if (b0 >= B) return;
    const int Hp = m.Hp;
    const bf16_t *Ot = static_cast<const bf16_t *>(m.Ot);
    const bf16_t *drow = static_cast<const bf16_t *>(m.d) + (size_t)(b0 + col) * Hp;
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int split = blockIdx.x;
    const int nblocks = m.Vp / 32;
    const int blk_begin = split * blocks_per_split;
    const int blk_end = min(nblocks, blk_begin + blocks_per_split);

    float mrun = FIXED ? m.m2_fixed : -INFINITY, srun = 0.f;
    for (int blk = blk_begin; blk < blk_end; ++blk) {
        const int v0 = blk * 32;
        const bf16_t *orow = Ot + (size_t)(v0 + col) * Hp;
        f32x16 acc = {0};
        for (int k0 = 8 * g; k0 < Hp; k0 += 16) {
            bf16x8 of = *reinterpret_cast<const bf16x8 *>(orow + k0);
            bf16x8 df = *reinterpret_cast<const bf16x8 *>(drow + k0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(of, df, acc, 0, 0, 0);
        }
        float x[16];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            f32x4 c = *reinterpret_cast<const f32x4 *>(cvec + v0 + 8 * q + 4 * g);
#pragma unroll
            for (int i = 0; i < 4; ++i) x[4 * q + i] = fmaf(acc[4 * q + i], kLog2e, c[i]);
        }
        lse2_accumulate16<FIXED>(x, mrun, srun);
    }
    // lanes l and l+32 hold the two halves of a row
    float m2 = __shfl_xor(mrun, 32, 64), s2 = __shfl_xor(srun, 32, 64);
    if (FIXED) srun += s2;
    else lse2_merge(mrun, srun, m2, s2);
    if (g == 0 && b0 + col < B) m.part[(size_t)(b0 + col) * kMaxSplits + split] = make_float2(mrun, srun);
}

// ------------------------------------------------------------------- plain fp32 ALU kernel
// A 64 (rows) x 64 (words) tile per workgroup of 256 threads, 4 x 4 logits per thread, K in
// chunks of 16 through LDS (stored k-major so a thread reads its four rows / four words as
// one 16-byte LDS access).
constexpr int kFM = 64, kFN = 64, kFK = 16;

template <bool FIXED>
__global__ __launch_bounds__(256) void outproj_plain_f32_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int blocks_per_split, int splits) {
    const int B = B_dev ? *B_dev : rows;
    const int b0 = blockIdx.y * kFM;
    if (b0 >= B) return;
    const int Hp = m.Hp;
    const float *Ot = static_cast<const float *>(m.Ot);
    const float *d = static_cast<const float *>(m.d);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int split = blockIdx.x;
    const int nblocks = m.Vp / kFN;
    const int blk_begin = split * blocks_per_split;
    const int blk_end = min(nblocks, blk_begin + blocks_per_split);

    __shared__ float As[kFK][kFM + 4];
    __shared__ float Bs[kFK][kFN + 4];
    __shared__ float2 red[kFM][16];
    const int t = threadIdx.x, tx = t & 15, ty = t >> 4;     // tx: word group, ty: row group
    const int lr = t >> 2, lk = (t & 3) * 4;                  // loader: row/word lr, k offset lk

    float mrun[4], srun[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { mrun[r] = FIXED ? m.m2_fixed : -INFINITY; srun[r] = 0.f; }

    for (int blk = blk_begin; blk < blk_end; ++blk) {
        const int v0 = blk * kFN;
        float acc[4][4];
        const f32x4 cv = *reinterpret_cast<const f32x4 *>(cvec + v0 + tx * 4);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
        for (int k0 = 0; k0 < Hp; k0 += kFK) {
            // rows of d beyond B are stale scratch; rows are independent, so whatever they
            // hold only reaches partials that are never written
            f32x4 av = *reinterpret_cast<const f32x4 *>(d + (size_t)(b0 + lr) * Hp + k0 + lk);
            f32x4 bv = *reinterpret_cast<const f32x4 *>(Ot + (size_t)(v0 + lr) * Hp + k0 + lk);
#pragma unroll
            for (int i = 0; i < 4; ++i) { As[lk + i][lr] = av[i]; Bs[lk + i][lr] = bv[i]; }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < kFK; ++k) {
                f32x4 a = *reinterpret_cast<const f32x4 *>(&As[k][ty * 4]);
                f32x4 b = *reinterpret_cast<const f32x4 *>(&Bs[k][tx * 4]);
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(a[r], b[c], acc[r][c]);
            }
            __syncthreads();
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            float x[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) x[c] = fmaf(acc[r][c], kLog2e, cv[c]);
            if (FIXED) {
#pragma unroll
                for (int c = 0; c < 4; ++c) srun[r] += fast_exp2(x[c]);
            } else {
                float mx = fmaxf(fmaxf(x[0], x[1]), fmaxf(x[2], x[3]));
                float mn = fmaxf(mrun[r], mx);
                if (mn != -INFINITY) {
                    float tsum = 0.f;
#pragma unroll
                    for (int c = 0; c < 4; ++c) tsum += fast_exp2(x[c] - mn);
                    srun[r] = srun[r] * fast_exp2(mrun[r] - mn) + tsum;
                    mrun[r] = mn;
                }
            }
        }
    }
    // combine the 16 word groups of every row, in a fixed order
#pragma unroll
    for (int r = 0; r < 4; ++r) red[ty * 4 + r][tx] = make_float2(mrun[r], srun[r]);
    __syncthreads();
    if (t < kFM) {
        float mm = red[t][0].x, ss = red[t][0].y;
        for (int i = 1; i < 16; ++i) {
            if (FIXED) ss += red[t][i].y;
            else lse2_merge(mm, ss, red[t][i].x, red[t][i].y);
        }
        if (b0 + t < B) m.part[(size_t)(b0 + t) * kMaxSplits + split] = make_float2(mm, ss);
    }
}

int choose_splits(int row_blocks, int col_blocks, int target_groups) {
    int s = (target_groups + row_blocks - 1) / row_blocks;
    if (s > kMaxSplits) s = kMaxSplits;
    if (s > col_blocks) s = col_blocks;
    if (s < 1) s = 1;
    return s;
}

}  // namespace

// defined in outproj_staged.hip
hipError_t launch_outproj_staged(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream);
// defined in outproj_tiled.hip
hipError_t launch_outproj_tiled(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                SplitInfo *splits, hipStream_t stream);

// defined in outproj_split3.hip
hipError_t launch_outproj_split3(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream);
// defined in outproj_rowstream.hip
hipError_t launch_outproj_rowstream(const ModelDev &m, int rows, const int *B_dev, SplitInfo *splits,
                                    hipStream_t stream);
// defined in outproj_stream.hip
hipError_t launch_outproj_stream(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream);

// Few rows: the time is the time to read the weights once (per launch: the streaming kernel holds
// 32 to 128 rows in LDS, depending on the model).  By itself up to 64 rows in at most two launches;
// on request up to 128 rows in at most four.
static bool stream_choice(const ModelDev &m, int rows, int kernel_choice) {
    const int per = outproj_stream_max_rows(m);
    if (per == 0) return false;
    const int launches = (rows + per - 1) / per;
    if (kernel_choice == 5) return rows <= 128 && launches <= 4;
    return kernel_choice == 0 && rows <= 64 && launches <= 2;
}

// Which bf16 kernel launch_outproj takes for a launch sized for `rows` rows.
enum Bf16Kernel { kBf16Stream, kBf16Staged, kBf16RowStream, kBf16Tiled, kBf16Plain };
static Bf16Kernel choose_bf16(const ModelDev &m, int rows, bool fixed_offset, int kernel_choice) {
    if (stream_choice(m, rows, kernel_choice)) return kBf16Stream;
    if (kernel_choice == 2 || (kernel_choice == 0 && outproj_staged_supported(m) && rows >= 128)) return kBf16Staged;
    // hidden sizes beyond the staged kernel's, batches and vocabularies that give every compute unit a
    // 256 x 256 tile, fixed offset: the hidden rows by-pass LDS (on request: any batch the model allows)
    const bool big = rows >= 256 && (long long)((rows + 255) / 256) * (m.Vp / 256) >= 256;
    if (fixed_offset && outproj_rowstream_supported(m) && (kernel_choice == 6 || (kernel_choice == 0 && big)))
        return kBf16RowStream;
    if (kernel_choice == 3 || kernel_choice == 6 || (kernel_choice == 0 && rows >= 64)) return kBf16Tiled;
    return kBf16Plain;
}

// Does the kernel launch_outproj will take read the row-ordered copy of the hidden block (m.d)?  The
// weight-streaming, staged and row-streaming kernels read the fragment-ordered one (m.dfrag) only, also
// when they fall back to weight streaming on the device; then the hidden update need not write m.d.
bool outproj_reads_row_order(const ModelDev &m, int rows, bool fixed_offset, int kernel_choice) {
    if (m.dtype != RNNLM_BF16) return true;
    const Bf16Kernel k = choose_bf16(m, rows, fixed_offset, kernel_choice);
    return k == kBf16Tiled || k == kBf16Plain;
}

// The kernel launch_outproj takes for these arguments, by the name a kernel trace shows.
const char *outproj_kernel_name(const ModelDev &m, int rows, bool fixed_offset, int kernel_choice) {
    if (m.dtype == RNNLM_BF16) {
        switch (choose_bf16(m, rows, fixed_offset, kernel_choice)) {
            case kBf16Stream: return "outproj_stream_kernel";
            case kBf16Staged: return "outproj_staged_kernel";
            case kBf16RowStream: return "outproj_rowstream_kernel";
            case kBf16Tiled: return "outproj_tiled_kernel";
            default: return "outproj_plain_bf16_kernel";
        }
    }
    if (stream_choice(m, rows, kernel_choice)) return "outproj_stream_kernel";
    if (kernel_choice == 3) return "outproj_tiled_kernel";
    if (m.Ot3 && (kernel_choice == 4 || (kernel_choice == 0 && rows >= 64))) return "outproj_split3_kernel";
    return "outproj_plain_f32_kernel";
}

hipError_t launch_outproj(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                          int kernel_choice, SplitInfo *splits, hipStream_t stream) {
    *splits = fixed_split_info(1);
    if (rows <= 0) return hipSuccess;
    if (m.dtype == RNNLM_BF16) {
        const Bf16Kernel which = choose_bf16(m, rows, fixed_offset, kernel_choice);
        if (which == kBf16Stream) return launch_outproj_stream(m, rows, B_dev, fixed_offset, splits, stream);
        if (which == kBf16Staged) return launch_outproj_staged(m, rows, B_dev, fixed_offset, splits, stream);
        if (which == kBf16RowStream) return launch_outproj_rowstream(m, rows, B_dev, splits, stream);
        if (which == kBf16Tiled) return launch_outproj_tiled(m, rows, B_dev, fixed_offset, splits, stream);
        const int row_groups = (rows + 127) / 128, col_blocks = m.Vp / 32;
        int S = choose_splits(row_groups, col_blocks, 1024);
        int per = (col_blocks + S - 1) / S;
        S = (col_blocks + per - 1) / per;
        dim3 grid(S, row_groups);
        if (fixed_offset)
            hipLaunchKernelGGL(outproj_plain_bf16_kernel<true>, grid, dim3(256), 0, stream, m, rows, B_dev, per, S);
        else
            hipLaunchKernelGGL(outproj_plain_bf16_kernel<false>, grid, dim3(256), 0, stream, m, rows, B_dev, per, S);
        *splits = fixed_split_info(S);
    } else {
        // fp32 on the bf16 matrix cores through the three-term split of both operands (six bf16
        // products per fp32 product at sixteen times the fp32 matrix rate, same accuracy): weight
        // streaming for few rows, the tiled three-term kernel from 64 rows on.  The tiled
        // fp32-MFMA kernel only on request; at the WSJ-sized workload it is no faster than the
        // FMA kernel below.
        if (stream_choice(m, rows, kernel_choice)) return launch_outproj_stream(m, rows, B_dev, fixed_offset, splits, stream);
        if (kernel_choice == 3) return launch_outproj_tiled(m, rows, B_dev, fixed_offset, splits, stream);
        if (m.Ot3 && (kernel_choice == 4 || (kernel_choice == 0 && rows >= 64)))
            return launch_outproj_split3(m, rows, B_dev, fixed_offset, splits, stream);
        const int row_groups = (rows + kFM - 1) / kFM, col_blocks = m.Vp / kFN;
        int S = choose_splits(row_groups, col_blocks, 1024);
        int per = (col_blocks + S - 1) / S;
        S = (col_blocks + per - 1) / per;
        dim3 grid(S, row_groups);
        if (fixed_offset)
            hipLaunchKernelGGL(outproj_plain_f32_kernel<true>, grid, dim3(256), 0, stream, m, rows, B_dev, per, S);
        else
            hipLaunchKernelGGL(outproj_plain_f32_kernel<false>, grid, dim3(256), 0, stream, m, rows, B_dev, per, S);
        *splits = fixed_split_info(S);
    }
    return hipGetLastError();
}

}  // namespace rnnlm
