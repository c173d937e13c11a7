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
//   - after the last chunk of a tile the logits are exponentiated and added.
// LDS rows are 128 bytes (8 chunks of 16); chunk c of row r sits at c ^ ((r >> 1) & 7), which
// spreads the 16 lanes served together by one ds_read_b128 over all 16 bank groups.
#include "device_utils.h"
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
template <typename T> struct Frag;
template <> struct Frag<bf16_t> { typedef bf16x8 type; };
template <> struct Frag<float> { typedef f32x4 type; };

template <int MB, int WN, int NS>
struct TiledCfg {
    static constexpr int kThreads = 2 * WN * 64;
    static constexpr int kWords = 64 * MB, kRows = 64 * WN;             // tile
    static constexpr int kWordBytes = kWords * 128, kRowBytes = kRows * 128;   // one chunk of each operand
    static constexpr int kStageBytes = kWordBytes + kRowBytes;
    static constexpr int kLdsBytes = NS * kStageBytes + 2 * kRows * 8;  // + final cross-wave reduction
    static constexpr int kWordLoads = kWords * 8 / kThreads, kRowLoads = kRows * 8 / kThreads;
    static_assert(kWords * 8 % kThreads == 0 && kRows * 8 % kThreads == 0, "whole loads per thread");
};

template <typename T, bool FIXED, int MB, int WN, int NS>
__global__ __launch_bounds__(2 * WN * 64) void outproj_tiled_kernel(ModelDev m, int rows,
                                                                    const int *__restrict__ B_dev, int RG,
                                                                    int S) {
    using C = TiledCfg<MB, WN, NS>;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int B = B_dev ? *B_dev : rows;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int rg = local % RG, split = xcd + kXcds * (local / RG);
    const int b0 = rg * C::kRows;
    if (b0 >= B) return;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;                  // word half, 64-row slice of the tile
    const int Hp = m.Hp;
    constexpr int kTK = 128 / (int)sizeof(T);                 // k per chunk
    typedef typename Frag<T>::type frag_t;
    const T *Ot = static_cast<const T *>(m.Ot);
    const T *D = static_cast<const T *>(m.d);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int ntiles = m.Vp / C::kWords;
    const int t_begin = (int)(((long long)split * ntiles) / S), t_end = (int)(((long long)(split + 1) * ntiles) / S);
    const int nk = Hp / kTK;                                  // chunks per tile
    const int nchunks = (t_end - t_begin) * nk;

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
    constexpr int kLoadsPerChunk = C::kWordLoads + C::kRowLoads;
    static_assert((NS - 2) * kLoadsPerChunk < 64, "vmcnt is a 6-bit counter");
#pragma unroll
    for (int c = 0; c < NS - 1; ++c)
        if (c < nchunks) issue(c, c);
    int stage = 0;
    for (int chunk = 0; chunk < nchunks; ++chunk) {
        // my loads of this chunk have landed: only the NS - 2 younger chunks may be outstanding
        // (near the end fewer are in flight: wait for everything)
        if (NS > 2 && chunk + NS - 2 < nchunks) wait_vmcnt<(NS - 2) * kLoadsPerChunk>();
        else wait_vmcnt<0>();
        __syncthreads();                                       // everybody's; the stage used last is free
        if (chunk + NS - 1 < nchunks) issue(chunk + NS - 1, stage == 0 ? NS - 1 : stage - 1);
        const int kc = chunk % nk;
        if (kc == 0) {
#pragma unroll
            for (int a = 0; a < MB; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b)
#pragma unroll
                    for (int i = 0; i < 16; ++i) acc[a][b][i] = 0.f;
        }
        const char *st = lds + stage * C::kStageBytes;
        stage = stage + 1 == NS ? 0 : stage + 1;
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
            __builtin_amdgcn_sched_barrier(0);                 // keep the reads ahead of the MFMAs
        }
        if (kc == nk - 1) {                                    // the tile is complete: exp-and-add
            const int v0 = (t_begin + chunk / nk) * C::kWords + wm * (32 * MB);
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
        }
    }
    // lanes l and l+32 hold two halves of a row; waves wm = 0, 1 hold the two word halves
    float2 *red = reinterpret_cast<float2 *>(lds + NS * C::kStageBytes);   // [2 (wm)][rows of the tile]
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
}

template <typename T, int MB, int WN, int NS>
hipError_t launch_tiled_shape(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, int wg_target,
                              SplitInfo *splits, hipStream_t stream) {
    using C = TiledCfg<MB, WN, NS>;
    static bool attr_set[2] = {false, false};
    const int which = fixed_offset ? 1 : 0;
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_tiled_kernel<T, true, MB, WN, NS>)
                                  : reinterpret_cast<const void *>(outproj_tiled_kernel<T, false, MB, WN, NS>);
    if (!attr_set[which]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, C::kLdsBytes);
        if (e != hipSuccess) return e;
        attr_set[which] = true;
    }
    const int RG = (rows + C::kRows - 1) / C::kRows, ntiles = m.Vp / C::kWords;
    // about wg_target workgroups; splits in multiples of 8 so that the row groups streaming the
    // same weights share an XCD; at most one split per tile, rounded UP to a multiple of 8 (a
    // few splits stay empty) so that no split gets two tiles while the others have one
    int Sx = wg_target / (kXcds * RG);
    if (Sx > (ntiles + kXcds - 1) / kXcds) Sx = (ntiles + kXcds - 1) / kXcds;
    if (Sx < 1) Sx = 1;
    if (Sx > kMaxSplits / kXcds) Sx = kMaxSplits / kXcds;
    const int S = kXcds * Sx;
    splits->fixed_splits = S;
    splits->staged_wg_per_xcd = 0;
    dim3 grid(kXcds * RG * Sx), block(C::kThreads);
    if (fixed_offset)
        hipLaunchKernelGGL((outproj_tiled_kernel<T, true, MB, WN, NS>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           RG, S);
    else
        hipLaunchKernelGGL((outproj_tiled_kernel<T, false, MB, WN, NS>), grid, block, C::kLdsBytes, stream, m, rows, B_dev,
                           RG, S);
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
            return launch_tiled_shape<bf16_t, 4, 4, 2>(m, rows, B_dev, fixed_offset, 256, splits, stream);
        // Batches that fill 256-row tiles, on a small vocabulary: one tile of 128 words x 256 rows
        // per workgroup, at most one workgroup per compute unit.  Such a workgroup lives for one
        // tile, a chain of load -> barrier -> use per chunk, and its compute unit pulls the bytes
        // in at its own limited rate: fewer bytes per workgroup than two 128 x 128 tiles (the
        // weights chunk is shared by all 256 rows), three stages (0 to 8 % faster, measured).
        const long long tall_tiles = (long long)((rows + 255) / 256) * (m.Vp / 128);
        if ((rows + 255) / 256 * 256 - rows <= 32 && tall_tiles <= 256)
            return launch_tiled_shape<bf16_t, 2, 4, 3>(m, rows, B_dev, fixed_offset, 256, splits, stream);
        return launch_tiled_shape<bf16_t, 2, 2, 2>(m, rows, B_dev, fixed_offset, 512, splits, stream);
    }
    return launch_tiled_shape<float, 2, 2, 2>(m, rows, B_dev, fixed_offset, 512, splits, stream);
}

}  // namespace rnnlm
