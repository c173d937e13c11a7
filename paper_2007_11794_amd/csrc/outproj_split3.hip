// Output projection + log-sum-exp for fp32 models on the bf16 matrix cores, at fp32 accuracy.
//
// Same result as the other output-projection kernels (normalising over all words of the
// vocabulary, Section 2.1 of the paper; the paper's models are fp32).  Every fp32 number is the
// exact sum of three bf16 numbers x = x1 + x2 + x3 (8 + 8 + 8 mantissa bits, each term rounded to
// nearest); of the nine cross terms of a product w d the six with the largest weight are kept
// (w1 d1, w1 d2, w2 d1, w1 d3, w3 d1, w2 d2; the dropped ones are below 2^-24 of the product) and
// added in the fp32 accumulators of the matrix instruction.
//
// Layout: weights and hidden block are kept term-interleaved in chunks of 32 units,
//     Ot3[v][j / 32][term][j % 32],   d3[b][j / 32][term][j % 32]      (bf16)
// so one chunk of the reduction is 192 contiguous bytes per row and every term is fetched once:
// 6 bytes per weight and launch (a layout that repeats the terms along a six times longer
// reduction, which would let a plain bf16 kernel do the job, moves twice as many bytes, and this
// contraction is bound by the bytes a compute unit can pull into LDS).
//   - a workgroup of 2 x WN waves owns 64 WN rows and walks the 128-word tiles of its vocabulary
//     split; a wave owns 64 words x 64 rows = 2 x 2 accumulators of 32x32;
//   - per chunk a stage holds 128 word rows + 64 WN hidden rows of 192 bytes, two stages, filled
//     by direct global->LDS loads;
//   - per 16 units a wave reads 6 A operands (2 word blocks x 3 terms) and 6 B operands (2 row
//     blocks x 3 terms) and issues 24 MFMA 32x32x16: one byte from LDS feeds twice the MFMAs it
//     would with repeated terms;
//   - MFMA roles as in the other kernels (A = words, B = rows): a lane holds sixteen logits of ONE
//     row per accumulator, the sum over words stays in the lane.
// LDS rows are 12 chunks of 16 bytes; logical chunk c of row r sits at (c + ((r >> 2) & 3)) % 12,
// which spreads the 16 lanes served together by one ds_read_b128 (16 consecutive rows, same c)
// over all 16 bank groups.  The direct loads write LDS linearly, so the rotation is applied on the
// global side: lane i fetches the chunk that belongs at position i.
#include "device_utils.h"
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kChunkUnits = 32;                  // fp32 units per chunk
constexpr int kRowLds = 3 * kChunkUnits * 2;     // 192 bytes per row and chunk
constexpr int kRowChunks = kRowLds / 16;         // 12

template <int WN>
struct Split3Cfg {
    static constexpr int kThreads = 2 * WN * 64;
    static constexpr int kWords = 128, kRows = 64 * WN;
    static constexpr int kWordBytes = kWords * kRowLds, kRowBytes = kRows * kRowLds;
    static constexpr int kStageBytes = kWordBytes + kRowBytes;
    static constexpr int kLdsBytes = 2 * kStageBytes + 2 * kRows * 8;   // + final cross-wave reduction
    static constexpr int kWordLoads = kWords * kRowChunks / kThreads, kRowLoads = kRows * kRowChunks / kThreads;
    static_assert(kWords * kRowChunks % kThreads == 0 && kRows * kRowChunks % kThreads == 0, "whole loads per thread");
    static_assert(kLdsBytes <= 160 * 1024, "");
};

__device__ __forceinline__ int lds_chunk_pos(int row, int c) { return (c + ((row >> 2) & 3)) % kRowChunks; }

template <bool FIXED, int WN>
__global__ __launch_bounds__(2 * WN * 64) void outproj_split3_kernel(ModelDev m, int rows,
                                                                     const int *__restrict__ B_dev, int wg_per_xcd,
                                                                     int sx_cap) {
    using C = Split3Cfg<WN>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // The split follows the TRUE number of rows (after the grouping of ids or the cache lookup only
    // the device knows it): few rows get many vocabulary splits, and the whole grid works.
    const int B = B_dev ? *B_dev : rows;
    if (B <= 0) return;                                       // uniform: no barrier is met
    const RowPlan plan = plan_rows(B, C::kRows, wg_per_xcd, sx_cap);
    const int S = plan.S, items = plan.RG * plan.Sx;
    // At most 64 rows after all: the time is then the time to read the weights once, and the first S
    // workgroups stream the fp32 weights instead (4 bytes per weight instead of 6, no LDS round trip
    // for them; eight-wave shape only, when the three terms of the hidden block fit this kernel's
    // LDS).  Same partials: split = workgroup index.
    if constexpr (C::kThreads == kStreamThreads) {
        if (B <= 64 && m.Ofrag) {
            const int KS = m.Hp >> 4;
            if (stream_lds_bytes(3, B <= 32 ? 1 : 2, KS) <= (size_t)C::kLdsBytes) {
                if ((int)blockIdx.x < S) {
                    if (B <= 32) outproj_stream_f32_body<1, FIXED>(m, B, 0, (int)blockIdx.x, S, lds);
                    else outproj_stream_f32_body<2, FIXED>(m, B, 0, (int)blockIdx.x, S, lds);
                }
                return;
            }
        }
    }
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;                  // word half, 64-row slice of the tile
    const int Hp = m.Hp;
    const size_t row_elems = (size_t)3 * Hp;                  // bf16 elements per row of Ot3 / d3
    const bf16_t *Ot3 = static_cast<const bf16_t *>(m.Ot3);
    const bf16_t *D3 = static_cast<const bf16_t *>(m.d3);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int ntiles = m.Vp / C::kWords;
    const int nk = Hp / kChunkUnits;                          // chunks per tile

    // loader: load q of this thread fills physical 16-byte chunk f = q * threads + tid of an operand
    // tile (row f / 12, position f % 12) with the logical chunk that belongs there
    constexpr int kMaxLoads = C::kWordLoads > C::kRowLoads ? C::kWordLoads : C::kRowLoads;
    uint32_t voff[kMaxLoads];
#pragma unroll
    for (int q = 0; q < kMaxLoads; ++q) {
        const int f = q * C::kThreads + tid;
        const int r = f / kRowChunks, p = f % kRowChunks;
        const int c = (p + kRowChunks - ((r >> 2) & 3)) % kRowChunks;
        voff[q] = (uint32_t)(r * (int)row_elems * 2 + c * 16);
    }
    const uint32_t wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = lds_address(lds);
    int aoff[2][3][2], boff[2][3][2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int t = 0; t < 3; ++t)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                // LDS offsets of this lane's operands: term t, k-step ks of a chunk = logical chunk 4 t + 2 ks + g
                const int ra = wm * 64 + h * 32 + col, rb = wn * 64 + h * 32 + col;
                aoff[h][t][ks] = ra * kRowLds + lds_chunk_pos(ra, 4 * t + 2 * ks + g) * 16;
                boff[h][t][ks] = C::kWordBytes + rb * kRowLds + lds_chunk_pos(rb, 4 * t + 2 * ks + g) * 16;
            }

    for (int item = local; item < items; item += wg_per_xcd) {
    const int rg = item % plan.RG, split = xcd + kXcds * (item / plan.RG);
    const int b0 = rg * C::kRows;
    const int t_begin = part_begin(split, ntiles, S), t_end = part_begin(split + 1, ntiles, S);
    const int nchunks = (t_end - t_begin) * nk;
    auto issue = [&](int chunk, int stage) {
        const int t = t_begin + chunk / nk, kc = chunk % nk;
        const bf16_t *wsrc = Ot3 + (size_t)t * C::kWords * row_elems + (size_t)kc * (3 * kChunkUnits);
        const bf16_t *dsrc = D3 + (size_t)b0 * row_elems + (size_t)kc * (3 * kChunkUnits);
        const uint32_t base = lds0 + stage * C::kStageBytes + wave_s * 1024;
#pragma unroll
        for (int q = 0; q < C::kWordLoads; ++q) lds_dma_16(wsrc, voff[q], base + q * (C::kThreads * 16));
#pragma unroll
        for (int q = 0; q < C::kRowLoads; ++q)
            lds_dma_16(dsrc, voff[q], base + C::kWordBytes + q * (C::kThreads * 16));
    };

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
        const char *st = lds + stage * C::kStageBytes;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            bf16x8 w[2][3], d[2][3];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int t = 0; t < 3; ++t) {
                    w[h][t] = *reinterpret_cast<const bf16x8 *>(st + aoff[h][t][ks]);
                    d[h][t] = *reinterpret_cast<const bf16x8 *>(st + boff[h][t][ks]);
                }
            // smallest cross terms first: (2,2) (3,1) (1,3) (2,1) (1,2) (1,1)
#pragma unroll
            for (int p = 0; p < 6; ++p) {
                constexpr int tw[6] = {1, 2, 0, 1, 0, 0}, td[6] = {1, 0, 2, 0, 1, 0};
#pragma unroll
                for (int a = 0; a < 2; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[a][tw[p]], d[b][td[p]], acc[a][b], 0, 0, 0);
            }
        }
        if (kc == nk - 1) {                                    // the tile is complete: exp-and-add
            const int v0 = (t_begin + chunk / nk) * C::kWords + wm * 64;
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
    float2 *red = reinterpret_cast<float2 *>(lds + 2 * C::kStageBytes);    // [2 (wm)][rows of the tile]
    __syncthreads();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const float m2 = __shfl_xor(mrun[h], 32, 64), s2 = __shfl_xor(srun[h], 32, 64);
        if (FIXED) srun[h] += s2;
        else lse2_merge(mrun[h], srun[h], m2, s2);
        if (g == 0) red[wm * C::kRows + wn * 64 + h * 32 + col] = make_float2(mrun[h], srun[h]);
    }
    __syncthreads();
    if (tid < C::kRows && b0 + tid < B) {
        float2 p = red[tid], q = red[C::kRows + tid];
        if (FIXED) p.y += q.y;
        else lse2_merge(p.x, p.y, q.x, q.y);
        m.part[(size_t)(b0 + tid) * kMaxSplits + split] = p;
    }
    }   // items
}

template <int WN>
hipError_t launch_split3_shape(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, SplitInfo *splits,
                               hipStream_t stream) {
    using C = Split3Cfg<WN>;
    static LdsLimit limit[2];
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_split3_kernel<true, WN>)
                                  : reinterpret_cast<const void *>(outproj_split3_kernel<false, WN>);
    if (hipError_t e = limit[fixed_offset ? 1 : 0].ensure(fn, C::kLdsBytes); e != hipSuccess) return e;
    // one workgroup per compute unit (a stage pair takes most of its LDS); at most one split per
    // tile of words, rounded UP to a multiple of 8 so that no split gets two tiles while the others
    // have one
    const int wg_per_xcd = 32, ntiles = m.Vp / C::kWords, sx_cap = (ntiles + kXcds - 1) / kXcds;
    *splits = SplitInfo{0, wg_per_xcd, C::kRows, sx_cap, 0};
    dim3 grid(kXcds * wg_per_xcd), block(C::kThreads);
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_split3_kernel<true, WN>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd, sx_cap);
    else
        hipLaunchKernelGGL((outproj_split3_kernel<false, WN>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd, sx_cap);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_outproj_split3(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream) {
    if (m.dtype != RNNLM_F32 || !m.Ot3 || !m.d3) return hipErrorInvalidValue;
    // 256-row tiles once the batch fills most of one, 128-row tiles below
    if (rows > 160) return launch_split3_shape<4>(m, rows, B_dev, fixed_offset, splits, stream);
    return launch_split3_shape<2>(m, rows, B_dev, fixed_offset, splits, stream);
}

}  // namespace rnnlm
