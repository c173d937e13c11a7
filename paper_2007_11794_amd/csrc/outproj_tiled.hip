// Output projection + log-sum-exp, LDS-tiled MFMA kernel for ANY hidden size, bf16 or fp32.
//
// Same result as the other output-projection kernels (normalising over all words of the
// vocabulary, Section 2.1 of the paper).  This is the form for models whose hidden block
// does not fit in registers (Hp > 512, e.g. the H = 1024 stress workload): both operands
// travel through LDS.
//   - a workgroup of 2 x WN waves owns TR = 64 WN rows and walks the TW = 64 MB-word tiles of
//     its vocabulary split; a wave owns 32 MB words x 64 rows = MB x 2 accumulators of 32x32.
//     Three shapes are built: 128 x 128 (4 waves, two workgroups per compute unit) for small
//     batches, 256 x 256 (8 waves) for batches of 256 rows and more, and 128 words x 256 rows
//     (8 waves) for such batches on a vocabulary too small to give every compute unit a
//     256 x 256 tile.  The kernel is bound by L2 -> LDS traffic (about 13 TB/s measured with
//     the small tile); the large tile moves half as many bytes per flop;
//   - the reduction length is cut in chunks of 128 bytes per row (64 bf16 or 32 fp32); a chunk
//     is TW rows of weights + TR rows of hidden values, in a ring of NS stages (two; three
//     for the 128 x 256 shape) filled by direct global->LDS loads;
//   - per 16-byte k-step a wave reads MB A operands (words) and two B operands (rows) and
//     issues 2 MB MFMA 32x32x16 (bf16), or 8 MB MFMA 32x32x2 (fp32, the full-precision matrix
//     instruction: one float per lane and operand, so a 16-byte read feeds four of them; lane
//     half g supplies k0 + 4 g + e to MFMA e, the same pairing for both operands);
//   - MFMA roles as in the staged kernel (A = words, B = rows): a lane holds sixteen logits
//     of ONE row per accumulator, the sum over words stays in the lane;
//   - the last chunk of a tile is taken accumulator by accumulator, and the exp-and-add of a
//     finished accumulator is interleaved with the MFMAs of the next one.
// LDS rows are 128 bytes (8 chunks of 16); chunk c of row r sits at c ^ ((r >> 1) & 7), which
// spreads the 16 lanes served together by one ds_read_b128 over all 16 bank groups.
#include "device_utils.h"
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

// MB accumulator rows x 2 accumulator columns += (MB A operands) x (2 B operands), 16 bytes of
// k per lane.
template <int MB>
__device__ __forceinline__ void mma_block(f32x16 (&acc)[MB][2], const bf16x8 (&a)[MB], const bf16x8 (&d)[2]) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], d[j], acc[i][j], 0, 0, 0);
}
template <int MB>
__device__ __forceinline__ void mma_block(f32x16 (&acc)[MB][2], const f32x4 (&a)[MB], const f32x4 (&d)[2]) {
#pragma unroll
    for (int e = 0; e < 4; ++e)
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i][e], d[j][e], acc[i][j], 0, 0, 0);
}
// One accumulator += one A operand x one B operand, 16 bytes of k per lane.
__device__ __forceinline__ void mma_one(f32x16 &acc, const bf16x8 &a, const bf16x8 &d) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, d, acc, 0, 0, 0);
}
__device__ __forceinline__ void mma_one(f32x16 &acc, const f32x4 &a, const f32x4 &d) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[e], d[e], acc, 0, 0, 0);
}
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { typedef bf16x8 type; };
template <> struct Frag<float> { typedef f32x4 type; };

template <int MB, int WN, int NS>
struct TiledCfg {
    static constexpr int kThreads = 2 * WN * 64;
    static constexpr int kWords = 64 * MB, kRows = 64 * WN;             // tile
    static constexpr int kWordBytes = kWords * 128, kRowBytes = kRows * 128;   // one chunk of each operand
    static constexpr int kStageBytes = kWordBytes + kRowBytes;
    static constexpr int kRedBytes = 2 * kRows * 8;                     // final cross-wave reduction
    static constexpr int kConstBytes = kWords * 4;                      // per stage: the constants of the chunk's tile
    static constexpr int kConstLanes = kWords / 4 / (2 * WN);           // lanes of a wave that fetch 16 bytes of them
    static constexpr int kLdsBytes = NS * kStageBytes + kRedBytes + NS * kConstBytes;
    static constexpr int kWordLoads = kWords * 8 / kThreads, kRowLoads = kRows * 8 / kThreads;
    static_assert(kWords * 8 % kThreads == 0 && kRows * 8 % kThreads == 0, "whole loads per thread");
    static_assert(kConstLanes >= 1 && kConstLanes * 4 * 2 * WN == kWords, "");
    static_assert(kLdsBytes <= 160 * 1024, "");
};

// OVL: the last chunk of a tile is taken accumulator by accumulator with the exp-and-add of the
// previous accumulator in between (about 10 % faster for the smaller tiles; the 256 x 256 tile,
// whose chunks wait for their loads anyway, is 1 % faster without: measured on one box).
template <typename T, bool FIXED, int MB, int WN, int NS, bool OVL>
__global__ __launch_bounds__(2 * WN * 64) void outproj_tiled_kernel(ModelDev m, int rows,
                                                                    const int *__restrict__ B_dev,
                                                                    int wg_per_xcd, int sx_cap, int stream_rows) {
    using C = TiledCfg<MB, WN, NS>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    // The split follows the TRUE number of rows (after the grouping of ids or the cache lookup only
    // the device knows it): few rows get many vocabulary splits, and the whole grid works.
    const int B = B_dev ? *B_dev : rows;
    if (B <= 0) return;                                       // uniform: no barrier is met
    // Very few rows after all (stream_rows: as many as this kernel's LDS holds over the whole
    // reduction length, 0 if the shape cannot do it): a tile would be a chain of 2 Hp / 128 load ->
    // barrier -> use steps on a fraction of the compute units; every workgroup streams its share
    // of the weights instead, split = workgroup index.
    if constexpr (sizeof(T) == 2 && C::kThreads == kStreamThreads) {
        if (B <= stream_rows) {
            if (B <= 32) outproj_stream_body<1, FIXED>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
            else outproj_stream_body<2, FIXED>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
            return;
        }
    }
    const RowPlan plan = plan_rows(B, C::kRows, wg_per_xcd, sx_cap);
    const int RG = plan.RG, S = plan.S, items = plan.RG * plan.Sx;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    // Hidden rows of all row groups beyond half an L2 (4 MB per XCD): the XCDs form P = 2 parts; part
    // p serves the row groups p RG/P .. (p+1) RG/P - 1 with all splits, split s on XCD
    // p + P (s % (8 / P)): the hidden rows one L2 has to keep shrink by P, the weights are fetched by
    // P XCDs (1.3 % at the stress workload; four or eight parts are slower, the weights cross the
    // fabric too often).
    const int P = (RG % 2 == 0 && (size_t)RG * C::kRows * m.Hp * sizeof(T) > ((size_t)2 << 20)) ? 2 : 1;
    const int RGp = RG / P, part = xcd % P;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;                  // word half, 64-row slice of the tile
    const int Hp = m.Hp;
    constexpr int kTK = 128 / (int)sizeof(T);                 // k per chunk
    typedef typename Frag<T>::type frag_t;
    const T *Ot = static_cast<const T *>(m.Ot);
    const T *D = static_cast<const T *>(m.d);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int ntiles = m.Vp / C::kWords;
    const int nk = Hp / kTK;                                  // chunks per tile

    // loader: load q of this thread fills physical 16-byte chunk f = q * threads + tid of an
    // operand tile (row f / 8, position f % 8) with the logical chunk that belongs there
    constexpr int kMaxLoads = C::kWordLoads > C::kRowLoads ? C::kWordLoads : C::kRowLoads;
    uint32_t voff[kMaxLoads];
#pragma unroll
    for (int q = 0; q < kMaxLoads; ++q) {
        const int f = q * C::kThreads + tid;
        const int r = f >> 3, p = f & 7, c = p ^ ((r >> 1) & 7);
        voff[q] = (uint32_t)(r * Hp * (int)sizeof(T) + c * 16);
    }
    const uint32_t wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = lds_address(lds);
    const char *const clds = lds + NS * C::kStageBytes + C::kRedBytes;   // constants, one slot per stage
    const uint32_t cl0 = lds_address(clds);
    for (int item = local; item < items; item += wg_per_xcd) {
    const int rg = part * RGp + item % RGp, split = xcd / P + (kXcds / P) * (item / RGp);
    const int b0 = rg * C::kRows;
    const int t_begin = part_begin(split, ntiles, S), t_end = part_begin(split + 1, ntiles, S);
    const int nchunks = (t_end - t_begin) * nk;
    auto issue = [&](int chunk, int stage) {
        const int t = t_begin + chunk / nk, k0 = (chunk % nk) * kTK;
        const T *wsrc = Ot + (size_t)t * C::kWords * Hp + k0;
        const T *dsrc = D + (size_t)b0 * Hp + k0;
        const uint32_t base = lds0 + stage * C::kStageBytes + wave_s * 1024;
#pragma unroll
        for (int q = 0; q < C::kWordLoads; ++q) lds_dma_16(wsrc, voff[q], base + q * (C::kThreads * 16));
#pragma unroll
        for (int q = 0; q < C::kRowLoads; ++q)
            lds_dma_16(dsrc, voff[q], base + C::kWordBytes + q * (C::kThreads * 16));
        // the per-word constants of the chunk's tile, every chunk (one more load per wave, so that
        // every wave counts the same number of loads per chunk)
        if (OVL && lane < C::kConstLanes)
            lds_dma_16(cvec + (size_t)t * C::kWords, (wave_s * C::kConstLanes + lane) * 16,
                       cl0 + stage * C::kConstBytes + wave_s * (C::kConstLanes * 16));
    };

    // LDS offsets of this lane's operands at k-step ks of a chunk: chunk index 2 ks + g of its row
    int aoff[MB][4], boff[2][4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
        for (int h = 0; h < MB; ++h) {
            const int ra = wm * (32 * MB) + h * 32 + col;
            aoff[h][ks] = ra * 128 + (((2 * ks + g) ^ ((ra >> 1) & 7)) * 16);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int rb = wn * 64 + h * 32 + col;
            boff[h][ks] = C::kWordBytes + rb * 128 + (((2 * ks + g) ^ ((rb >> 1) & 7)) * 16);
        }
    }

    float mrun[2], srun[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) { mrun[h] = FIXED ? m.m2_fixed : -INFINITY; srun[h] = 0.f; }
    f32x16 acc[MB][2];

    // ring of NS stages: NS - 1 chunks are on their way while one is being used
    constexpr int kLoadsPerChunk = C::kWordLoads + C::kRowLoads + (OVL ? 1 : 0);
    static_assert((NS - 2) * kLoadsPerChunk < 64, "vmcnt is a 6-bit counter");
#pragma unroll
    for (int c = 0; c < NS - 1; ++c)
        if (c < nchunks) issue(c, c);
    int stage = 0, chunk = 0;
    // Start of a chunk's use: its loads have landed for everybody, the stage used last is free and
    // takes the chunk NS - 1 ahead.  Returns the chunk's stage.
    auto begin_chunk = [&]() -> int {
        // my loads of this chunk have landed: only the NS - 2 younger chunks may be outstanding
        // (near the end fewer are in flight: wait for everything)
        if (NS > 2 && chunk + NS - 2 < nchunks) wait_vmcnt<(NS - 2) * kLoadsPerChunk>();
        else wait_vmcnt<0>();
        __syncthreads();
        if (chunk + NS - 1 < nchunks) issue(chunk + NS - 1, stage == 0 ? NS - 1 : stage - 1);
        const int cur = stage;
        stage = stage + 1 == NS ? 0 : stage + 1;
        ++chunk;
        return cur;
    };
    // Tile by tile; the accumulators live from the top of this loop body to its bottom only (a
    // straight line: the chunks but the last in an inner loop, then the last one), which lets the
    // compiler keep each of them in one place.
    for (int t = t_begin; t < t_end; ++t) {
#pragma unroll
        for (int a = 0; a < MB; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b)
#pragma unroll
                for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        for (int kc = 0; kc < nk - 1; ++kc) {
            const char *st = lds + begin_chunk() * C::kStageBytes;
            // operands of k-step ks+1 are requested before the MFMAs of k-step ks are issued
            frag_t fa[2][MB], fd[2][2];
#pragma unroll
            for (int h = 0; h < MB; ++h) fa[0][h] = *reinterpret_cast<const frag_t *>(st + aoff[h][0]);
#pragma unroll
            for (int h = 0; h < 2; ++h) fd[0][h] = *reinterpret_cast<const frag_t *>(st + boff[h][0]);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks + 1 < 4) {
#pragma unroll
                    for (int h = 0; h < MB; ++h)
                        fa[(ks + 1) & 1][h] = *reinterpret_cast<const frag_t *>(st + aoff[h][ks + 1]);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        fd[(ks + 1) & 1][h] = *reinterpret_cast<const frag_t *>(st + boff[h][ks + 1]);
                }
                mma_block<MB>(acc, fa[ks & 1], fd[ks & 1]);
                __builtin_amdgcn_sched_barrier(0);             // keep the reads ahead of the MFMAs
            }
        }
        if (!OVL) {
            // last chunk as the others, then the exp-and-add of the whole tile
            const char *st = lds + begin_chunk() * C::kStageBytes;
            frag_t fa[2][MB], fd[2][2];
#pragma unroll
            for (int h = 0; h < MB; ++h) fa[0][h] = *reinterpret_cast<const frag_t *>(st + aoff[h][0]);
#pragma unroll
            for (int h = 0; h < 2; ++h) fd[0][h] = *reinterpret_cast<const frag_t *>(st + boff[h][0]);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                if (ks + 1 < 4) {
#pragma unroll
                    for (int h = 0; h < MB; ++h)
                        fa[(ks + 1) & 1][h] = *reinterpret_cast<const frag_t *>(st + aoff[h][ks + 1]);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
                        fd[(ks + 1) & 1][h] = *reinterpret_cast<const frag_t *>(st + boff[h][ks + 1]);
                }
                mma_block<MB>(acc, fa[ks & 1], fd[ks & 1]);
                __builtin_amdgcn_sched_barrier(0);
            }
            const int v0 = t * C::kWords + wm * (32 * MB);
#pragma unroll
            for (int a = 0; a < MB; ++a) {
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
        } else {
            // Last chunk of the tile: accumulator by accumulator (all four k-steps of one, then the
            // next), so that a finished accumulator's exp-and-add runs in the shadow of the next
            // one's MFMAs; only the last of the 2 MB accumulators is finished in the open.
            const int cur_stage = begin_chunk();
            const char *st = lds + cur_stage * C::kStageBytes;
            const float *cl = reinterpret_cast<const float *>(clds + cur_stage * C::kConstBytes) + wm * (32 * MB) + 4 * g;
            frag_t fa1[2], fd1[2];
            f32x4 cprev[4];
#pragma unroll
            for (int idx = 0; idx < 2 * MB; ++idx) {
                const int b = idx / MB, a = idx % MB;
                const int pi = idx > 0 ? idx - 1 : 0, pb = pi / MB, pa = pi % MB;   // the accumulator finished just before
                fa1[0] = *reinterpret_cast<const frag_t *>(st + aoff[a][0]);
                fd1[0] = *reinterpret_cast<const frag_t *>(st + boff[b][0]);
                if (idx > 0) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) cprev[q] = *reinterpret_cast<const f32x4 *>(cl + pa * 32 + 8 * q);
                }
                float x[16];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    if (ks + 1 < 4) {
                        fa1[(ks + 1) & 1] = *reinterpret_cast<const frag_t *>(st + aoff[a][ks + 1]);
                        fd1[(ks + 1) & 1] = *reinterpret_cast<const frag_t *>(st + boff[b][ks + 1]);
                    }
                    mma_one(acc[a][b], fa1[ks & 1], fd1[ks & 1]);
                    if (idx > 0) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            x[4 * ks + i] = fmaf(acc[pa][pb][4 * ks + i], kLog2e, cprev[ks][i]);
                            if (FIXED) srun[pb] += fast_exp2(x[4 * ks + i]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (!FIXED && idx > 0) lse2_fold16<false>(x, mrun[pb], srun[pb]);
            }
            {
                float x[16];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 c = *reinterpret_cast<const f32x4 *>(cl + (MB - 1) * 32 + 8 * q);
#pragma unroll
                    for (int i = 0; i < 4; ++i) x[4 * q + i] = fmaf(acc[MB - 1][1][4 * q + i], kLog2e, c[i]);
                }
                lse2_fold16<FIXED>(x, mrun[1], srun[1]);
            }
        }
    }
    // lanes l and l+32 hold two halves of a row; waves wm = 0, 1 hold the two word halves
    float2 *red = reinterpret_cast<float2 *>(lds + NS * C::kStageBytes);   // [2 (wm)][rows of the tile]; kRedBytes
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

template <typename T, int MB, int WN, int NS, bool OVL>
hipError_t launch_tiled_shape(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, int wg_target,
                              SplitInfo *splits, hipStream_t stream) {
    using C = TiledCfg<MB, WN, NS>;
    static LdsLimit limit[2];
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_tiled_kernel<T, true, MB, WN, NS, OVL>)
                                  : reinterpret_cast<const void *>(outproj_tiled_kernel<T, false, MB, WN, NS, OVL>);
    if (hipError_t e = limit[fixed_offset ? 1 : 0].ensure(fn, C::kLdsBytes); e != hipSuccess) return e;
    // wg_target workgroups; at most one split per tile of words, rounded UP to a multiple of 8 (a few
    // splits stay empty) so that no split gets two tiles while the others have one
    const int wg_per_xcd = wg_target / kXcds, ntiles = m.Vp / C::kWords, sx_cap = (ntiles + kXcds - 1) / kXcds;
    // rows the weight-streaming body can take inside this kernel: 64 or 32, as its LDS allows
    int stream_rows = 0;
    if (sizeof(T) == 2 && C::kThreads == kStreamThreads && m.Ofrag && kXcds * wg_per_xcd <= kMaxSplits) {
        const int KS = m.Hp >> 4;
        if (stream_lds_bytes(1, 2, KS) <= (size_t)C::kLdsBytes) stream_rows = 64;
        else if (stream_lds_bytes(1, 1, KS) <= (size_t)C::kLdsBytes) stream_rows = 32;
    }
    *splits = SplitInfo{0, wg_per_xcd, C::kRows, sx_cap, stream_rows};
    dim3 grid(kXcds * wg_per_xcd), block(C::kThreads);
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_tiled_kernel<T, true, MB, WN, NS, OVL>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd, sx_cap, stream_rows);
    else
        hipLaunchKernelGGL((outproj_tiled_kernel<T, false, MB, WN, NS, OVL>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           wg_per_xcd, sx_cap, stream_rows);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_outproj_tiled(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                SplitInfo *splits, hipStream_t stream) {
    if (m.dtype == RNNLM_BF16) {
        // 256 x 256 tiles, one workgroup per compute unit, once batch and vocabulary give every
        // compute unit such a tile; smaller problems fill the chip better with 128 x 128
        const long long big_tiles = (long long)((rows + 255) / 256) * (m.Vp / 256);
        if (rows >= 256 && big_tiles >= 256)
            return launch_tiled_shape<bf16_t, 4, 4, 2, false>(m, rows, B_dev, fixed_offset, 256, splits, stream);
        // Batches that fill 256-row tiles, on a small vocabulary: one tile of 128 words x 256 rows
        // per workgroup, at most one workgroup per compute unit.  Such a workgroup lives for one
        // tile, a chain of load -> barrier -> use per chunk, and its compute unit pulls the bytes
        // in at its own limited rate: fewer bytes per workgroup than two 128 x 128 tiles (the
        // weights chunk is shared by all 256 rows), three stages (0 to 8 % faster, measured).
        const long long tall_tiles = (long long)((rows + 255) / 256) * (m.Vp / 128);
        if ((rows + 255) / 256 * 256 - rows <= 32 && tall_tiles <= 256)
            return launch_tiled_shape<bf16_t, 2, 4, 3, true>(m, rows, B_dev, fixed_offset, 256, splits, stream);
        return launch_tiled_shape<bf16_t, 2, 2, 2, true>(m, rows, B_dev, fixed_offset, 512, splits, stream);
    }
    return launch_tiled_shape<float, 2, 2, 2, true>(m, rows, B_dev, fixed_offset, 512, splits, stream);
}

}  // namespace rnnlm
