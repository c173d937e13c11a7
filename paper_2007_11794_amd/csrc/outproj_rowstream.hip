// Output projection + log-sum-exp, bf16 MFMA kernel for hidden sizes beyond what the staged kernel
// keeps in registers (Hp > 512; the H = 1024 stress workload), batches of 256 rows and more, fixed
// log-sum-exp offset.
//
// Same result as the other output-projection kernels (normalising over all words of the vocabulary,
// Section 2.1 of the paper).  The LDS-tiled kernel sends BOTH operands through LDS; two stages of
// 64 KB fill it, so a chunk's loads have less than one chunk's time to land, and the launch waits
// for them 40 % of the time.  Here only the weights go through LDS:
//   - a workgroup (8 waves) owns 256 rows and walks the 256-word tiles of its vocabulary split; a
//     wave owns 32 ROWS and all 256 words of the tile: eight 32x32 accumulators (128 VGPRs), eight
//     independent MFMA chains;
//   - the reduction length is cut in chunks of 64 (128 bytes per word row); a chunk of weights is
//     32 KB, four LDS stages, filled by direct global->LDS loads three chunks ahead;
//   - the wave's rows of the hidden block come from the fragment-ordered copy (one MFMA B operand =
//     1 KB contiguous, already multiplied by log2 e) straight into registers by loads the compiler
//     does not track, one chunk (four operands) ahead; nothing of them touches LDS;
//   - one barrier per chunk, in the MIDDLE of its 32 MFMAs (it publishes the next chunk and frees
//     the stage of the one before); the loads are issued one by one between the MFMAs; every wave
//     issues the same loads in the same order, so all vmcnt immediates are compile-time figures
//     (dummy loads past the end of the split keep that true);
//   - MFMA roles as in the staged kernel (A = words from LDS, B = rows from registers): a lane holds
//     sixteen logits of ONE row per accumulator, the sum over words stays in the lane.  With the
//     fixed offset the accumulators start from the tile's constants and end as base-2 logits; the
//     exp-and-add of a finished tile is done block by block in front of the first MFMA that
//     overwrites the block in the next tile's first chunk.
// LDS rows are 128 bytes (8 pieces of 16); piece c of row r sits at c ^ ((r >> 1) & 7), which spreads
// the 16 lanes served together by one ds_read_b128 over all bank groups (as in the tiled kernel).
#include <type_traits>

#include "device_utils.h"
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kThreads = 512;
constexpr int kWords = 256, kRows = 256;                 // tile of a workgroup
constexpr int kBlocks = kWords / 32;                     // 32-word blocks = accumulators per wave
constexpr int kStages = 4;
constexpr int kStageBytes = kWords * 128;                // one chunk of weights
constexpr int kConstBytes = kWords * 4;                  // the tile's constants travel with every chunk
constexpr int kLdsBytes = kStages * (kStageBytes + kConstBytes);
constexpr int kWeightLoads = kWords * 8 / kThreads;      // direct-to-LDS loads per thread and chunk
constexpr int kDmaPerChunk = kWeightLoads + 1;           // + the constants
constexpr int kDOperands = 4;                            // B operands per wave and chunk
constexpr int kMfmaPerChunk = kBlocks * kDOperands;      // 32
constexpr int kPrefetch = 4;                             // A operands read this many MFMAs ahead
static_assert(kWeightLoads == 4 && kMfmaPerChunk == 32, "the issue slots below are written for these");

template <int BEGIN, int END, typename Fn>
__device__ __forceinline__ void static_for(Fn &&fn) {
    if constexpr (BEGIN < END) {
        fn(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(fn);
    }
}

// A B operand requested without the compiler knowing that a load is in flight (see the staged
// kernel): the register counts as defined at once and stays unread until await_operand.
template <int OFFSET>
__device__ __forceinline__ void load_operand(bf16x8 &dst, const bf16_t *lane_ptr) {
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(lane_ptr), "n"(OFFSET) : "memory");
}
template <int YOUNGER>
__device__ __forceinline__ void await_operand(bf16x8 &op) {
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(op) : "n"(YOUNGER));
}
// lds_dma_16 by the first eight lanes of the wave only (128 bytes), without a branch.
__device__ __forceinline__ void lds_dma_16_lanes8(const void *sbase, uint32_t voff, uint32_t lds_base) {
    uint64_t saved_exec;
    asm volatile("s_mov_b64 %0, exec\n\ts_mov_b64 exec, 0xff\n\tglobal_load_lds_dwordx4 %2, %3\n\ts_mov_b64 exec, %0"
                 : "=&s"(saved_exec)
                 : "{m0}"(lds_base), "v"(voff), "s"(sbase)
                 : "memory");
}

__global__ __launch_bounds__(kThreads) void outproj_rowstream_kernel(ModelDev m, int rows,
                                                                     const int *__restrict__ B_dev, int wg_per_xcd,
                                                                     int sx_cap, int stream_rows) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int B = B_dev ? *B_dev : rows;
    if (B <= 0) return;                                       // uniform: no barrier is met
    // very few rows after all: every workgroup streams its share of the weights (as the tiled kernel)
    static_assert(kThreads == kStreamThreads, "");
    if (B <= stream_rows) {
        if (B <= 32) outproj_stream_body<1, true>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
        else outproj_stream_body<2, true>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
        return;
    }
    const RowPlan plan = plan_rows(B, kRows, wg_per_xcd, sx_cap);
    const int RG = plan.RG, S = plan.S, items = plan.RG * plan.Sx;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    // hidden rows of all row groups beyond half an L2: the XCDs form two parts that serve half of the
    // row groups each (as in the tiled kernel)
    const int P = (RG % 2 == 0 && (size_t)RG * kRows * m.Hp * 2 > ((size_t)2 << 20)) ? 2 : 1;
    const int RGp = RG / P, part = xcd % P;
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Hp = m.Hp, KS = Hp >> 4, nk = Hp >> 6;          // nk: chunks per tile
    const bf16_t *Ot = static_cast<const bf16_t *>(m.Ot);
    const float *cvec = m.cvec2_fixed;
    const int ntiles = m.Vp / kWords;
    const uint32_t lds0 = lds_address(lds), cl0 = lds0 + kStages * kStageBytes;
    const char *const clds = lds + kStages * kStageBytes;

    // loader: load q of this thread fills physical 16-byte piece f = q * threads + tid of a stage
    // (word row f / 8, position f % 8) with the logical piece that belongs there
    uint32_t voff[kWeightLoads];
#pragma unroll
    for (int q = 0; q < kWeightLoads; ++q) {
        const int f = q * kThreads + tid, r = f >> 3, p = f & 7, c = p ^ ((r >> 1) & 7);
        voff[q] = (uint32_t)(r * Hp * 2 + c * 16);
    }
    // this lane's A operand at k-step ks of a chunk, block 0: piece 2 ks + g of word row `col`
    int aoff[kDOperands];
#pragma unroll
    for (int ks = 0; ks < kDOperands; ++ks) aoff[ks] = col * 128 + (((2 * ks + g) ^ ((col >> 1) & 7)) * 16);

    for (int item = local; item < items; item += wg_per_xcd) {
        const int rg = part * RGp + item % RGp, split = xcd / P + (kXcds / P) * (item / RGp);
        const int t_begin = part_begin(split, ntiles, S), t_end = part_begin(split + 1, ntiles, S);
        const int nchunks = (t_end - t_begin) * nk;
        const int b = rg * kRows + wave * 32 + col;           // this lane's row
        if (nchunks <= 0) {                                   // uniform: an empty split adds nothing
            if (g == 0 && b < B) m.part[(size_t)b * kMaxSplits + split] = make_float2(m.m2_fixed, 0.f);
            continue;
        }
        // this lane's 16 bytes of B operand 0 of its wave's rows; operand ks lies ks KB further on
        const bf16_t *dfr = static_cast<const bf16_t *>(m.dfrag) + ((size_t)(rg * (kRows / 32) + wave) * KS * 64 + lane) * 8;

        // ---- what the loop carries
        int c = 0;                                            // chunk in use
        int kc_next = nk > 1 ? 1 : 0;                         // k-chunk of chunk c + 1
        int it = t_begin, ikc = 0;                            // tile and k-chunk of the next chunk to request
        int ic = 0;                                           // ... and its number
        // Direct-to-LDS loads of the next chunk to request, one piece per call; past the end of the
        // split: dummies (same count for vmcnt, one cache line of the weights' first bytes).
        const bf16_t *wsrc = Ot;
        const float *csrc = cvec;
        bool real = true;
        uint32_t wdst = 0, cdst = 0;
        auto next_request = [&]() __attribute__((always_inline)) {
            real = ic < nchunks;
            wsrc = Ot + (real ? (size_t)it * kWords * Hp + (size_t)ikc * 64 : (size_t)0);
            csrc = cvec + (real ? it * kWords : 0);
            wdst = lds0 + (ic & (kStages - 1)) * kStageBytes + wave * 1024;
            cdst = cl0 + (ic & (kStages - 1)) * kConstBytes + wave * 128;
            ++ic;
            const bool wrap = ikc + 1 == nk;
            ikc = wrap ? 0 : ikc + 1;
            it += wrap ? 1 : 0;
        };
        auto request_piece = [&](int q) __attribute__((always_inline)) {
            if (q < kWeightLoads) lds_dma_16(wsrc, real ? voff[q] : 0u, wdst + q * (kThreads * 16));
            else lds_dma_16_lanes8(csrc, (uint32_t)(wave * 8 + lane) * 16, cdst);
        };

        // ---- prologue: chunks 0 and 1, the B operands of chunk 0, chunk 2
        bf16x8 dop[kDOperands], dnext[kDOperands];
        next_request();
#pragma unroll
        for (int q = 0; q < kDmaPerChunk; ++q) request_piece(q);
        next_request();
#pragma unroll
        for (int q = 0; q < kDmaPerChunk; ++q) request_piece(q);
        load_operand<0>(dop[0], dfr);
        load_operand<1024>(dop[1], dfr);
        load_operand<2048>(dop[2], dfr);
        load_operand<3072>(dop[3], dfr);
        next_request();
#pragma unroll
        for (int q = 0; q < kDmaPerChunk; ++q) request_piece(q);
        // chunks 0 and 1 and the operands have landed once only chunk 2 is outstanding
        static_for<0, kDOperands>([&](auto j) __attribute__((always_inline)) { await_operand<kDmaPerChunk>(dop[decltype(j)::value]); });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        next_request();                                       // chunk 3: requested by chunk 0's second half

        f32x16 acc[kBlocks];
#pragma unroll
        for (int blk = 0; blk < kBlocks; ++blk) {
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[blk][i] = -INFINITY;      // "previous tile" of the first: adds 2^-inf = 0
            // opaque to the compiler: otherwise it specialises the first tile on the constant (twice the
            // code, and the constants spilled around it)
            asm volatile("" : "+v"(acc[blk]));
        }
        float srun = 0.f;
        bf16x8 a[kPrefetch];
#pragma unroll
        for (int i = 0; i < kPrefetch; ++i)
            a[i] = *reinterpret_cast<const bf16x8 *>(lds + i * 4096 + aoff[0]);      // MFMA i of a chunk: block i, k-step 0

        // One chunk: MFMA i is block i % 8, k-step i / 8.  first (first chunk of a tile): in front of
        // a block's first MFMA the block's old contents (the finished logits of the tile before) go
        // through exp-and-add and the block restarts from the tile's constants.
        //
        // Loads of a wave per chunk, in program order (the slot is the MFMA they follow):
        //   d0'@1  d1'@5  d2'@9  d3'@13  [barrier before MFMA 16]  w0@17  w1@20  w2@23  w3@26  c@29
        // dk' = B operand k of the NEXT chunk into a second set of registers (moved over at the end of
        // the chunk: a full chunk of time to arrive), w0..w3, c = weights and constants of chunk c+3 into
        // the stage of chunk c-1.  Nine loads.  The barrier waits for chunk c+1, whose last load (c@29 of
        // chunk c-2) is followed by the nine of chunk c-1 and four of this one: 13.  At the end of the
        // chunk the next operands have landed once only this chunk's five direct-to-LDS loads are
        // outstanding.  The prologue's order and its wait (everything but chunk 2 landed) give chunk 0
        // counts that are no larger.
        auto chunk = [&](bool first) __attribute__((always_inline)) {
            const char *stage = lds + (c & (kStages - 1)) * kStageBytes;
            const char *next_stage = lds + ((c + 1) & (kStages - 1)) * kStageBytes;
            const float *cst = reinterpret_cast<const float *>(clds + (c & (kStages - 1)) * kConstBytes) + 4 * g;
            const bf16_t *dnext_ptr = dfr + (size_t)kc_next * 2048;
            static_for<0, kMfmaPerChunk>([&](auto step) __attribute__((always_inline)) {
                constexpr int i = decltype(step)::value, blk = i % kBlocks, ks = i / kBlocks;
                if constexpr (i == 16) {
                    wait_vmcnt<13>();
                    asm volatile("" ::: "memory");
                    __builtin_amdgcn_s_barrier();
                    asm volatile("" ::: "memory");
                }
                const bf16x8 cur = a[i % kPrefetch];
                {
                    constexpr int n = i + kPrefetch, nb = n % kMfmaPerChunk % kBlocks, nks = n % kMfmaPerChunk / kBlocks;
                    const char *st = n < kMfmaPerChunk ? stage : next_stage;
                    a[i % kPrefetch] = *reinterpret_cast<const bf16x8 *>(st + nb * 4096 + aoff[nks]);
                }
                if (ks == 0 && first) {                        // uniform; the only branches of the chunk body
#pragma unroll
                    for (int e = 0; e < 16; ++e) srun += fast_exp2(acc[blk][e]);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x4 cn = *reinterpret_cast<const f32x4 *>(cst + blk * 32 + 8 * q);
#pragma unroll
                        for (int e = 0; e < 4; ++e) acc[blk][4 * q + e] = cn[e];
                    }
                }
                acc[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, dop[ks], acc[blk], 0, 0, 0);
                if constexpr (i == 1) load_operand<0>(dnext[0], dnext_ptr);
                if constexpr (i == 5) load_operand<1024>(dnext[1], dnext_ptr);
                if constexpr (i == 9) load_operand<2048>(dnext[2], dnext_ptr);
                if constexpr (i == 13) load_operand<3072>(dnext[3], dnext_ptr);
                if constexpr (i >= 17 && i <= 29 && (i - 17) % 3 == 0) request_piece((i - 17) / 3);
                __builtin_amdgcn_sched_barrier(0);             // keep the LDS reads ahead of their MFMAs
            });
            static_for<0, kDOperands>([&](auto j) __attribute__((always_inline)) {
                await_operand<kDmaPerChunk>(dnext[decltype(j)::value]);
                dop[decltype(j)::value] = dnext[decltype(j)::value];
            });
            next_request();
            ++c;
            kc_next = kc_next + 1 == nk ? 0 : kc_next + 1;
        };

        // ONE loop over the chunks of all tiles with ONE body: with the tile's first chunk as a second
        // instantiation in an outer loop the compiler kept the accumulators in different registers per
        // loop level and paid with hundreds of copies and spills (whose scratch traffic would also
        // have broken the hand-counted vmcnt).
        int kc_cur = 0;
        for (int cc = 0; cc < nchunks; ++cc) {
            chunk(kc_cur == 0);
            kc_cur = kc_cur + 1 == nk ? 0 : kc_cur + 1;
        }
        // the last tile's logits
#pragma unroll
        for (int blk = 0; blk < kBlocks; ++blk)
#pragma unroll
            for (int e = 0; e < 16; ++e) srun += fast_exp2(acc[blk][e]);
        srun += __shfl_xor(srun, 32, 64);                     // lanes l and l+32 hold the two halves of a row
        if (g == 0 && b < B) m.part[(size_t)b * kMaxSplits + split] = make_float2(m.m2_fixed, srun);
        wait_vmcnt<0>();                                      // dummy loads may still be in flight
        __syncthreads();                                      // LDS is reused by the next item
    }
}

}  // namespace

bool outproj_rowstream_supported(const ModelDev &m) {
    return m.dtype == RNNLM_BF16 && m.dfrag != nullptr;
}

hipError_t launch_outproj_rowstream(const ModelDev &m, int rows, const int *B_dev, SplitInfo *splits,
                                    hipStream_t stream) {
    static LdsLimit limit;
    const void *fn = reinterpret_cast<const void *>(outproj_rowstream_kernel);
    if (hipError_t e = limit.ensure(fn, kLdsBytes); e != hipSuccess) return e;
    // one workgroup per compute unit; at most one split per tile of words, rounded UP to a multiple of 8
    const int wg_per_xcd = 32, ntiles = m.Vp / kWords, sx_cap = (ntiles + kXcds - 1) / kXcds;
    int stream_rows = 0;                                      // rows the weight-streaming body can take in this LDS
    if (m.Ofrag) {
        const int KS = m.Hp >> 4;
        if (stream_lds_bytes(1, 2, KS) <= (size_t)kLdsBytes) stream_rows = 64;
        else if (stream_lds_bytes(1, 1, KS) <= (size_t)kLdsBytes) stream_rows = 32;
    }
    *splits = SplitInfo{0, wg_per_xcd, kRows, sx_cap, stream_rows};
    hipLaunchKernelGGL(outproj_rowstream_kernel, dim3(kXcds * wg_per_xcd), dim3(kThreads), kLdsBytes, stream, m, rows, B_dev,
                       wg_per_xcd, sx_cap, stream_rows);
    return hipGetLastError();
}

}  // namespace rnnlm
