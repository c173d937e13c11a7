// Output projection + log-sum-exp, LDS-staged bf16 MFMA kernel for Hp in {128, 256, 512}.
//
// What is computed is the same as in the plain kernel (normalising over all words of the
// vocabulary, Section 2.1 of the paper); this is the fast form for batches of >= 128 rows.
//
// Shape of the work.  The hidden block d = h' - 1/2 is tiny (rows x Hp bf16, 1 MB at
// 1024 x 512) and the output weights Ot[Vp][Hp] are large (64 MB at V = 65536), so the
// weights are streamed exactly once per row group and the hidden block never moves:
//   - a workgroup (8 waves) owns 256 rows; each wave keeps ITS 32 rows of d for the whole
//     reduction length in registers (Hp/16 MFMA B-operands, 128 VGPRs at Hp = 512), loaded from
//     the fragment-ordered copy of the block (one operand = 1 KB contiguous), which holds
//     d * log2(e): the accumulators are base-2 logits;
//   - the weights of 32 words (32 x Hp bf16, 32 KB at Hp = 512) form one LDS stage; four
//     stages are filled round-robin by direct global->LDS loads (no VGPR round trip), two to
//     three blocks ahead of use;
//   - per block a wave issues Hp/16 chained MFMA 32x32x16: A = 32 words x 16 k from LDS
//     (read four steps ahead), B = 16 k x 32 rows from registers, so lane l holds 16 logits
//     of ONE row and the sum over words stays inside the lane;
//   - the exp-and-add of block i is interleaved, instruction by instruction, with the MFMAs
//     of block i+1, so the vector ALU works in the shadow of the matrix core (the unrolled
//     block body is kept free of branches for that: see staged_block_fixed / staged_block);
//   - one workgroup barrier per block.  It publishes the landing of block i+1 while block i
//     is being computed, so no wave ever waits at a barrier for data it is about to use, and
//     the first operands of block i+1 are already in registers when block i ends.
// With the fixed log-sum-exp offset (the usual case) nothing at all happens at the boundary
// between two blocks: the barrier sits in the MIDDLE of a block's MFMA chain (a wave that waits
// there has its last MFMA in the pipe, and the chain goes on without any hand-over), the loads of
// block i+3 are issued one by one between the MFMAs of the block's second half instead of in a
// burst behind the barrier, two accumulator sets alternate (no copy between blocks, the next chain
// does not wait for the last MFMA of this one), and the constants a chain starts from are read
// from LDS into the resting accumulator set half a block before they are needed.
// LDS rows are XOR-swizzled in 16-byte chunks (chunk c of word r sits at c ^ (r & 15)) so
// that the 16 lanes served together by one ds_read_b128 hit 16 different bank groups.  The
// direct loads write LDS linearly (lane i -> base + 16 i), so the swizzle is applied on the
// global side: lane i fetches the chunk that belongs at position i.
//
// When the batch turns out to hold at most 64 rows (the count may be known on the device only),
// the kernel runs the weight-streaming body instead (outproj_stream_body.h): see the top of
// the kernel.
//
// Work split (staged_plan): workgroup id modulo 8 is the XCD; vocabulary split s runs on
// XCD s % 8, with all row groups of that split next to each other, so the row groups that
// stream the same weights hit in the same 4 MB L2 and HBM is read once.
#include <type_traits>

#include "device_utils.h"
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kThreads = 512;
constexpr int kStages = 4;
constexpr int kCSlots = 8;                       // ring of per-block constants (32 floats each)
constexpr int kCSlotBytes = kStagedWords * 4;
constexpr int kPrefetch = 4;                     // A operands read this many k-steps ahead

template <int HP>
struct StagedCfg {
    static constexpr int KS = HP / 16;                       // MFMA k-steps per block
    static constexpr int CPR = HP / 8;                       // 16-byte chunks per word row
    static constexpr int kStageChunks = kStagedWords * CPR;
    static constexpr int kStageBytes = kStageChunks * 16;
    static constexpr int kLoadsPerThread = kStageChunks / kThreads;     // weight loads per block
    static constexpr int kLoadsPerBlock = kLoadsPerThread + 1;          // + one for the constants
    static constexpr int kLdsBytes = kStages * kStageBytes + kCSlots * kCSlotBytes;
    static_assert(kStageChunks % kThreads == 0, "stage must be a whole number of loads per thread");
    static_assert(CPR >= 16, "swizzle needs at least 16 chunks per row");
    static_assert(kLoadsPerBlock <= 6, "s_waitcnt immediates below assume few loads per block");
};

// Per-thread constants of the block loader.
template <int HP>
struct Loader {
    uint32_t voff[StagedCfg<HP>::kLoadsPerThread];           // byte offset in the block of words
    uint32_t wave;                                           // wave index, in an SGPR
    int lane;
    __device__ __forceinline__ void init() {
        using C = StagedCfg<HP>;
        const int tid = threadIdx.x;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        lane = tid & 63;
#pragma unroll
        for (int q = 0; q < C::kLoadsPerThread; ++q) {
            const int f = q * kThreads + tid;                // physical chunk this lane fills
            const int r = f / C::CPR, p = f % C::CPR;
            const int c = p ^ (r & 15);                      // logical chunk that belongs there
            voff[q] = (uint32_t)(r * HP * 2 + c * 16);
        }
    }
    // Start the loads of the 32-word block whose first word is v0 into stage / constant slot.
    __device__ __forceinline__ void issue(const bf16_t *Ot, const float *cvec, int v0, uint32_t stage_lds,
                                          uint32_t cslot_lds) const {
        using C = StagedCfg<HP>;
        const bf16_t *blk = Ot + (size_t)v0 * HP;
#pragma unroll
        for (int q = 0; q < C::kLoadsPerThread; ++q)
            lds_dma_16(blk, voff[q], stage_lds + (q * kThreads + wave * 64) * 16);
        // the 32 constants of the block: 16 bytes per wave, by its lane 0
        if (lane == 0) lds_dma_16(cvec + v0, wave * 16, cslot_lds + wave * 16);
    }
    // The same in pieces and without branches (the fixed-offset block body is one basic block):
    // weight load q of the block, and its constants.  real = false turns the load into a dummy
    // that counts like a real one for vmcnt but fetches the first bytes of the weights (always
    // there, one cache line for the whole wave) into the same, free, LDS stage.
    __device__ __forceinline__ void issue_weights(const bf16_t *blk, int q, bool real, uint32_t stage_lds) const {
        lds_dma_16(blk, real ? voff[q] : 0u, stage_lds + (q * kThreads + wave * 64) * 16);
    }
    __device__ __forceinline__ void issue_consts(const float *cblk, uint32_t cslot_lds) const {
        lds_dma_16_lane0(cblk, wave * 16, cslot_lds + wave * 16);
    }
    __device__ __forceinline__ void issue_all(const bf16_t *Ot, const float *cvec, int v0, bool real,
                                              uint32_t stage_lds, uint32_t cslot_lds) const {
        using C = StagedCfg<HP>;
        const int v = real ? v0 : 0;
        const bf16_t *blk = Ot + (size_t)v * HP;
#pragma unroll
        for (int q = 0; q < C::kLoadsPerThread; ++q) issue_weights(blk, q, real, stage_lds);
        issue_consts(cvec + v, cslot_lds);
    }
};

// The hidden block arrives multiplied by log2(e) (fragment-ordered copy), so the accumulators
// are base-2 already.  Fixed offset: the accumulators START at the block's constants, and a
// finished accumulator IS the logit (one VALU instruction less per logit; |constant| < 100 there,
// so accumulating on top of it costs nothing the tolerance would notice).  Running maximum
// (constants of any size): the constants are added at the end, x = acc + c2.
template <bool FIXED>
__device__ __forceinline__ void finish_logits(const f32x16 &acc, const f32x4 *cn, int g, float (&x)[16]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        f32x4 c = {0.f, 0.f, 0.f, 0.f};
        if (!FIXED) c = cn[2 * q + g];
#pragma unroll
        for (int i = 0; i < 4; ++i) x[4 * q + i] = FIXED ? acc[4 * q + i] : acc[4 * q + i] + c[i];
    }
}

#define RNNLM_A_FRAG(stage, ks) \
    (*reinterpret_cast<const bf16x8 *>((stage) + aoff[(ks) & 7] + ((ks) >> 3) * 256))

// One 32-word block for this wave's 32 rows.
//   stage      LDS stage of this block; a[] already holds its first kPrefetch A operands
//   next_stage LDS stage of the following block (after the last block: any stage, the operands
//              read from it are not used); on return a[] holds ITS first kPrefetch A operands
//              -- that block was published one barrier earlier.  Never a branch here: the
//              unrolled body must stay ONE basic block, or the compiler sinks the exp-and-add
//              of the previous block out of the MFMA sequence into the last block
//   ccur       this block's constants (fixed offset: the accumulators start from them)
//   pacc, pcn  the previous block's raw accumulators and its constants: its exp-and-add is
//              spread over this block's k-steps (fixed offset) or done up front (running max)
template <int HP, bool FIXED>
__device__ __forceinline__ void staged_block(const char *stage, const char *next_stage, const int (&aoff)[8],
                                             bf16x8 (&a)[kPrefetch], const bf16x8 (&dreg)[HP / 16], int g,
                                             const f32x4 *ccur, f32x16 &pacc, const f32x4 *pcn, float &mrun,
                                             float &srun) {
    constexpr int KS = HP / 16;
    static_assert(KS >= 2 * kPrefetch, "");
    f32x16 acc = {0};
    if (FIXED) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 c = ccur[2 * q + g];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[4 * q + i] = c[i];
        }
    } else {
        float x[16];
        finish_logits<false>(pacc, pcn, g, x);
        lse2_fold16<false>(x, mrun, srun);
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const bf16x8 cur = a[ks % kPrefetch];
        if (ks + kPrefetch < KS) a[ks % kPrefetch] = RNNLM_A_FRAG(stage, ks + kPrefetch);
        else a[ks % kPrefetch] = RNNLM_A_FRAG(next_stage, ks + kPrefetch - KS);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, dreg[ks], acc, 0, 0, 0);
        if (FIXED) {
            // sixteen logits of the previous block spread evenly over the KS steps
#pragma unroll
            for (int e = 0; e < 16; ++e)
                if ((e * KS) / 16 == ks) srun += fast_exp2(pacc[e]);
        }
        // keep this order: the compiler's scheduler would otherwise sink every LDS read to
        // just before its MFMA and expose the LDS latency on each step
        __builtin_amdgcn_sched_barrier(0);
    }
    pacc = acc;
}

// One MFMA B operand (this lane's 16 bytes of a 1 KB fragment) requested WITHOUT the compiler
// knowing that a load is in flight: the register is defined for it at once, and the caller keeps
// it unread until await_d_operand has waited for the data.  (A load the compiler can see makes
// it guard the operand with vmcnt waits of its own inside the block loop, and those drain the
// direct-to-LDS loads, which it cannot see.)
template <int OFFSET>
__device__ __forceinline__ void load_d_operand(bf16x8 &dst, const bf16_t *lane_ptr) {
    static_assert(OFFSET >= 0 && OFFSET < 4096, "immediate offset of a global load");
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=v"(dst) : "v"(lane_ptr), "n"(OFFSET) : "memory");
}
// Wait until at most `younger` of this wave's vector-memory operations are outstanding; the
// operand goes in and out so that its first use cannot move in front of the wait.
template <int YOUNGER>
__device__ __forceinline__ void await_d_operand(bf16x8 &op) {
    static_assert(YOUNGER >= 0 && YOUNGER < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%1)" : "+v"(op) : "n"(YOUNGER));
}
// fn(std::integral_constant<int, I>) for I = BEGIN .. END - 1, in order.
template <int BEGIN, int END, typename Fn>
__device__ __forceinline__ void static_for(Fn &&fn) {
    if constexpr (BEGIN < END) {
        fn(std::integral_constant<int, BEGIN>{});
        static_for<BEGIN + 1, END>(fn);
    }
}

// Dispatch of load_d_operand on a compile-time operand index: operand j of a wave lies 1 KB behind
// operand j - 1; one pointer every 4 KB, immediate offsets in between.
template <int J>
__device__ __forceinline__ void load_d_operand_at(bf16x8 &dst, const bf16_t *dfr) {
    load_d_operand<(J % 4) * 1024>(dst, dfr + (size_t)(J / 4) * 2048);
}

// What block 0 of an item issues besides its own work (staged_block_fixed<HP, true>): the part of
// d that the prologue has not requested, and blocks 1 and 2.  All loads of a wave are issued in
// one fixed program order, so the number of loads younger than any given one is a compile-time
// figure: that is what the vmcnt immediates of block 0 are computed from.
template <int HP>
struct FirstBlockSchedule {
    using C = StagedCfg<HP>;
    static constexpr int KS = C::KS, HALF = KS / 2, L = C::kLoadsPerBlock, NW = C::kLoadsPerThread;
    static constexpr int kLoadStep = (HALF - 2) / NW;
    static constexpr int D0 = KS < 8 ? KS : 8;                 // operands of d requested by the prologue
    static_assert(2 * L <= HALF, "blocks 1 and 2 are requested in the first half of block 0");
    // loads issued in k-step k: before its MFMA an operand of d (e1) and a load of block 1 or 2 (e2),
    // after its MFMA the regular loads of block 3 (e3)
    static constexpr int e1(int k) { return k + D0 < KS ? 1 : 0; }
    static constexpr int e2(int k) { return k < 2 * L ? 1 : 0; }
    static constexpr int e3(int k) {
        int n = (k == KS - 2) ? 1 : 0;
        for (int q = 0; q < NW; ++q)
            if (k == HALF + 1 + q * kLoadStep) ++n;
        return n;
    }
    // loads younger than operand ks of d when the MFMA of k-step ks is about to be issued
    static constexpr int younger_than_d(int ks) {
        int n = 0;
        if (ks < D0) {
            n = D0 - 1 - ks;
            for (int k = 0; k <= ks; ++k) n += e1(k) + e2(k);
            for (int k = 0; k < ks; ++k) n += e3(k);
        } else {
            const int j0 = ks - D0;                             // the k-step that requested it
            n = e2(j0);
            for (int k = j0 + 1; k <= ks; ++k) n += e1(k) + e2(k);
            for (int k = j0; k < ks; ++k) n += e3(k);
        }
        return n;
    }
    // loads younger than the last load of block 1 (k-step L - 1) at the barrier on top of k-step HALF
    static constexpr int younger_than_block1() {
        int n = 0;
        for (int k = L; k < HALF; ++k) n += e1(k) + e2(k);
        for (int k = L - 1; k < HALF; ++k) n += e3(k);
        return n;
    }
    static constexpr int worst() {
        int w = younger_than_block1();
        for (int ks = 0; ks < KS; ++ks)
            if (younger_than_d(ks) > w) w = younger_than_d(ks);
        return w;
    }
    static_assert(worst() < 64, "vmcnt is a 6-bit counter");
};
struct FirstBlockLoads {
    const bf16_t *dfr;          // this lane's 16 bytes of operand 0 of its wave's rows
    const bf16_t *blk[2];       // weights of blocks 1 and 2 (or the dummy source)
    const float *cst[2];        // their constants
    bool real[2];
    uint32_t stage[2], cslot[2];
};

// Fixed offset: one 32-word block for this wave's 32 rows, as ONE basic block.
//   acc     on entry the block's constants (the base-2 logits start from them), on return the
//           finished logits of the block
//   other   on entry the finished logits of the previous block (-inf before the first): their
//           exp-and-add is spread over the first half of the k-steps; on return the constants of
//           block bi+1 (read from the ring in the second half; after the last block: a landed
//           slot, unused)
// Half way through, the barrier publishes block bi+1 (everybody's loads of it have landed: the
// only younger loads of a wave are those of block bi+2) and frees the stage of block bi-1, which
// takes block bi+3 (past the end of the split: dummy loads, so that every wave always has the same
// number of loads in flight and the vmcnt immediates hold).  On return a[] holds the first
// kPrefetch A operands of block bi+1.
//
// FIRST (block 0 of an item): the prologue has requested block 0 and the first operands of d only,
// so that the chain starts early; the rest of d is requested here, one operand per k-step eight
// k-steps ahead of its use, and blocks 1 and 2 load by load in the first half.  Every MFMA waits
// for ITS operand of d alone, and the barrier for block 1 alone (FirstBlockSchedule has the
// counts): the chain runs at the pace at which d arrives instead of starting after all of it.
template <int HP, bool FIRST>
__device__ __forceinline__ void staged_block_fixed(const char *lds, const char *cring, uint32_t lds0,
                                                   uint32_t cring0, const Loader<HP> &loader, const bf16_t *Ot,
                                                   const float *cvec, int blk0, int nblk, int bi,
                                                   const int (&aoff)[8], bf16x8 (&a)[kPrefetch],
                                                   bf16x8 (&dreg)[HP / 16], int g, f32x16 &acc,
                                                   f32x16 &other, float &srun, const FirstBlockLoads &first) {
    using C = StagedCfg<HP>;
    using F = FirstBlockSchedule<HP>;
    constexpr int KS = C::KS, HALF = KS / 2, NW = C::kLoadsPerThread;
    constexpr int kLoadStep = (HALF - 2) / NW;                 // k-steps between two weight loads
    static_assert(KS >= 2 * kPrefetch && kLoadStep >= 1 && HALF + 1 + (NW - 1) * kLoadStep < KS - 2, "");
    const char *stage = lds + (bi & 3) * C::kStageBytes;
    const char *next_stage = lds + (((bi + 1 < nblk) ? bi + 1 : bi) & 3) * C::kStageBytes;
    const f32x4 *cnext = reinterpret_cast<const f32x4 *>(cring + ((bi + 1) & 7) * kCSlotBytes);
    const bool real = bi + 3 < nblk;
    const int v3 = real ? (blk0 + bi + 3) * kStagedWords : 0;
    const bf16_t *blk3 = Ot + (size_t)v3 * HP;
    const uint32_t stage3 = lds0 + ((bi + 3) & 3) * C::kStageBytes, cslot3 = cring0 + ((bi + 3) & 7) * kCSlotBytes;
    // the k-steps as a compile-time loop: every condition below is a constant, and so are the vmcnt
    // immediates
    static_for<0, KS>([&](auto step) __attribute__((always_inline)) {
        constexpr int ks = decltype(step)::value;
        if constexpr (ks == HALF) {
            if constexpr (FIRST) wait_vmcnt<F::younger_than_block1()>();
            else wait_vmcnt<C::kLoadsPerBlock>();
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
        }
        const bf16x8 cur = a[ks % kPrefetch];
        if constexpr (ks + kPrefetch < KS) a[ks % kPrefetch] = RNNLM_A_FRAG(stage, ks + kPrefetch);
        else a[ks % kPrefetch] = RNNLM_A_FRAG(next_stage, ks + kPrefetch - KS);
        if constexpr (FIRST) {
            if constexpr (ks + F::D0 < KS) load_d_operand_at<ks + F::D0>(dreg[ks + F::D0], first.dfr);
            if constexpr (ks < F::L) {
                if constexpr (ks < NW) loader.issue_weights(first.blk[0], ks, first.real[0], first.stage[0]);
                else loader.issue_consts(first.cst[0], first.cslot[0]);
            } else if constexpr (ks < 2 * F::L) {
                if constexpr (ks - F::L < NW) loader.issue_weights(first.blk[1], ks - F::L, first.real[1], first.stage[1]);
                else loader.issue_consts(first.cst[1], first.cslot[1]);
            }
            await_d_operand<F::younger_than_d(ks)>(dreg[ks]);
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, dreg[ks], acc, 0, 0, 0);
        // the previous block's sixteen logits, over k-steps 1 .. HALF
#pragma unroll
        for (int e = 0; e < 16; ++e)
            if (1 + (e * HALF) / 16 == ks) srun += fast_exp2(other[e]);
        // second half: loads of block bi+3, constants of block bi+1 into the resting accumulators
#pragma unroll
        for (int q = 0; q < NW; ++q)
            if (ks == HALF + 1 + q * kLoadStep) loader.issue_weights(blk3, q, real, stage3);
        if constexpr (ks == KS - 2) loader.issue_consts(cvec + v3, cslot3);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            if (ks == HALF + 1 + (q * (HALF - 1)) / 4) {
                const f32x4 c = cnext[2 * q + g];
#pragma unroll
                for (int i = 0; i < 4; ++i) other[4 * q + i] = c[i];
            }
        // keep this order: the compiler's scheduler would otherwise sink every LDS read to
        // just before its MFMA and expose the LDS latency on each step
        __builtin_amdgcn_sched_barrier(0);
    });
}

// Fixed offset: all blocks of one (row group, split) item for this wave's rows; returns the sum
// of 2^(logit - offset) over the item's words for this lane's half of its row.
template <int HP>
__device__ __forceinline__ float staged_item_fixed(const ModelDev &m, char *lds, char *cring, const Loader<HP> &loader,
                                                   const int (&aoff)[8], int rg, int blk0, int nblk, int wave,
                                                   int lane, int g) {
    using C = StagedCfg<HP>;
    constexpr int KS = C::KS;
    const bf16_t *Ot = static_cast<const bf16_t *>(m.Ot);
    const float *cvec = m.cvec2_fixed;
    const uint32_t lds0 = lds_address(lds), cring0 = lds_address(cring);
    // Block 0 and the first operands of this wave's rows of d (all k of 32 rows are MFMA B operands
    // held in registers; rows beyond B hold stale scratch: rows are independent and those lanes'
    // results are dropped).  The rest of d and blocks 1 and 2 are requested by block 0 itself.
    using F = FirstBlockSchedule<HP>;
    loader.issue_all(Ot, cvec, blk0 * kStagedWords, true, lds0, cring0);
    bf16x8 dreg[KS];
    FirstBlockLoads first;
    // fragment (row block, ks) of the fragment-ordered copy: 64 lanes x 16 bytes in a row
    first.dfr = static_cast<const bf16_t *>(m.dfrag) + ((size_t)(rg * (kStagedRows / 32) + wave) * KS * 64 + lane) * 8;
    static_for<0, F::D0>([&](auto j) __attribute__((always_inline)) {
        load_d_operand_at<decltype(j)::value>(dreg[decltype(j)::value], first.dfr);
    });
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        first.real[i] = i + 1 < nblk;
        const int v = first.real[i] ? (blk0 + i + 1) * kStagedWords : 0;
        first.blk[i] = Ot + (size_t)v * HP;
        first.cst[i] = cvec + v;
        first.stage[i] = lds0 + (i + 1) * C::kStageBytes;
        first.cslot[i] = cring0 + (i + 1) * kCSlotBytes;
    }
    // Block 0 has landed once only the younger loads are outstanding: the first operands of d.
    wait_vmcnt<F::D0>();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();                             // block 0 is published
    asm volatile("" ::: "memory");
    // From block 1 on every wave has, at the barrier in the middle of block bi, the loads of blocks
    // bi+1 and bi+2 in flight at most.
    bf16x8 a[kPrefetch];
#pragma unroll
    for (int i = 0; i < kPrefetch; ++i) a[i] = RNNLM_A_FRAG(lds, i);
    f32x16 acc0, acc1;
    {
        const f32x4 *c0 = reinterpret_cast<const f32x4 *>(cring);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 c = c0[2 * q + g];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc0[4 * q + i] = c[i];
        }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) acc1[i] = -INFINITY;        // "previous block" of block 0: adds 2^-inf = 0
    float srun = 0.f;
#define RNNLM_BLOCK(FIRST, BI, ACC, OTHER) \
    staged_block_fixed<HP, FIRST>(lds, cring, lds0, cring0, loader, Ot, cvec, blk0, nblk, BI, aoff, a, dreg, g, ACC, OTHER, srun, first)
    RNNLM_BLOCK(true, 0, acc0, acc1);
    int bi = 1;
    for (; bi + 1 < nblk; bi += 2) {
        RNNLM_BLOCK(false, bi, acc1, acc0);
        RNNLM_BLOCK(false, bi + 1, acc0, acc1);
    }
    if (bi < nblk) {
        RNNLM_BLOCK(false, bi, acc1, acc0);
#pragma unroll
        for (int e = 0; e < 16; ++e) srun += fast_exp2(acc1[e]);
    } else {
#pragma unroll
        for (int e = 0; e < 16; ++e) srun += fast_exp2(acc0[e]);
    }
#undef RNNLM_BLOCK
    // dummy loads may still be in flight into stages the next item fills first
    wait_vmcnt<0>();
    return srun;
}

template <int HP, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_staged_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev,
                                                                  int wg_per_xcd) {
    using C = StagedCfg<HP>;
    constexpr int KS = C::KS;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    char *const cring = lds + kStages * C::kStageBytes;
    const int B = B_dev ? *B_dev : rows;
    if (B <= 0) return;                                       // uniform: nothing to do, no barrier met
    // Few rows after all (after the grouping or the cache lookup only the device knows how many
    // are left): the time is then the time to read the weights once, and the workgroup streams
    // them instead.  Same grid, and the same partials come out: with one row group the vocabulary
    // is cut into as many splits as there are workgroups, split = workgroup index.
    static_assert(kThreads == kStreamThreads, "");
    static_assert(C::kLdsBytes >= 2 * KS * 1024 + kStreamWaves * 64 * 8, "LDS for two row blocks of the streaming form");
    if (B <= 64 && m.Ofrag && (int)gridDim.x == staged_plan(B, wg_per_xcd).S) {
        if (B <= 32) outproj_stream_body<1, FIXED>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
        else outproj_stream_body<2, FIXED>(m, B, 0, (int)blockIdx.x, (int)gridDim.x, lds);
        return;
    }
    const StagedPlan plan = staged_plan(B, wg_per_xcd);
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const bf16_t *Ot = static_cast<const bf16_t *>(m.Ot);
    const float *cvec = FIXED ? m.cvec2_fixed : m.cvec2;
    const int T = m.Vp / kStagedWords;                       // 32-word blocks in the vocabulary
    const int items = plan.RG * plan.Sx;
    const uint32_t lds0 = lds_address(lds), cring0 = lds_address(cring);
    Loader<HP> loader;
    loader.init();
    // Swizzled LDS offsets of this lane's A operand: chunk (2 ks + g) of word `col`.  Only the
    // low 4 bits of the chunk index take part in the swizzle, so eight per-lane offsets
    // (aoff[ks % 8]) plus compile-time constants cover all k-steps.
    int aoff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) aoff[j] = col * (C::CPR * 16) + ((((2 * j) | g) ^ (col & 15)) * 16);

    for (int item = local; item < items; item += wg_per_xcd) {
        const int rg = item % plan.RG, split = xcd + kXcds * (item / plan.RG);
        const int blk0 = part_begin(split, T, plan.S);
        const int nblk = part_begin(split + 1, T, plan.S) - blk0;
        const int b = rg * kStagedRows + wave * 32 + col;     // this lane's row
        if (FIXED) {
            float srun = 0.f;
            if (nblk > 0) srun = staged_item_fixed<HP>(m, lds, cring, loader, aoff, rg, blk0, nblk, wave, lane, g);
            srun += __shfl_xor(srun, 32, 64);                 // lanes l and l+32 hold the two halves of a row
            if (g == 0 && b < B) m.part[(size_t)b * kMaxSplits + split] = make_float2(m.m2_fixed, srun);
            __syncthreads();                                  // LDS is reused by the next item
            continue;
        }

        // Blocks 0 and 1 first, then this wave's rows of d (all k, as MFMA B operands; rows
        // beyond B hold stale scratch: rows are independent and those lanes' results are dropped).
#pragma unroll
        for (int i = 0; i < 2; ++i)
            if (i < nblk)
                loader.issue(Ot, cvec, (blk0 + i) * kStagedWords, lds0 + i * C::kStageBytes, cring0 + i * kCSlotBytes);
        bf16x8 dreg[KS];
        {
            // fragment (row block, ks) of the fragment-ordered copy: 64 lanes x 16 bytes in a row
            const bf16_t *dfr = static_cast<const bf16_t *>(m.dfrag) +
                                ((size_t)(rg * (kStagedRows / 32) + wave) * KS * 64 + lane) * 8;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) dreg[ks] = *reinterpret_cast<const bf16x8 *>(dfr + (size_t)ks * 512);
        }
        float mrun = FIXED ? m.m2_fixed : -INFINITY, srun = 0.f;
        // raw accumulators of the previous block, still to be exponentiated; -inf adds 2^-inf = 0
        f32x16 pacc;
#pragma unroll
        for (int i = 0; i < 16; ++i) pacc[i] = -INFINITY;

        // Blocks 0 and 1 have landed once at most the KS younger loads of d are outstanding; d
        // itself is awaited operand by operand as the first block's MFMAs consume it.
        wait_vmcnt<(KS < 64 ? KS : 63)>();
        __syncthreads();                                      // blocks 0 and 1 are published
#pragma unroll
        for (int i = 2; i < 4; ++i)
            if (i < nblk)
                loader.issue(Ot, cvec, (blk0 + i) * kStagedWords, lds0 + i * C::kStageBytes, cring0 + i * kCSlotBytes);

        bf16x8 a[kPrefetch];
        if (nblk > 0) {
#pragma unroll
            for (int i = 0; i < kPrefetch; ++i) a[i] = RNNLM_A_FRAG(lds, i);
        }
        for (int bi = 0; bi < nblk; ++bi) {
            if (bi > 0) {
                // Publish block bi+1: my loads of it have landed (the only younger ones are
                // those of block bi+2), then everybody's.  Everybody is also done with block
                // bi-1, so its stage takes block bi+3.
                if (bi + 2 < nblk) wait_vmcnt<C::kLoadsPerBlock>();
                else wait_vmcnt<0>();
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
                if (bi + 3 < nblk)
                    loader.issue(Ot, cvec, (blk0 + bi + 3) * kStagedWords, lds0 + ((bi + 3) & 3) * C::kStageBytes,
                                 cring0 + ((bi + 3) & 7) * kCSlotBytes);
            }
            const char *stage = lds + (bi & 3) * C::kStageBytes;
            const char *next_stage = lds + (((bi + 1 < nblk) ? bi + 1 : bi) & 3) * C::kStageBytes;
            // constants of the previous block (for block 0 any landed slot: its pacc is -inf)
            const f32x4 *pcn = reinterpret_cast<const f32x4 *>(cring + ((bi ? bi - 1 : 0) & 7) * kCSlotBytes);
            const f32x4 *ccur = reinterpret_cast<const f32x4 *>(cring + (bi & 7) * kCSlotBytes);
            staged_block<HP, FIXED>(stage, next_stage, aoff, a, dreg, g, ccur, pacc, pcn, mrun, srun);
        }
        if (nblk > 0) {                                       // the last block's exp-and-add
            float x[16];
            finish_logits<FIXED>(pacc, reinterpret_cast<const f32x4 *>(cring + ((nblk - 1) & 7) * kCSlotBytes), g, x);
            lse2_fold16<FIXED>(x, mrun, srun);
        }
        // lanes l and l+32 hold the two halves of a row
        const float m2 = __shfl_xor(mrun, 32, 64), s2 = __shfl_xor(srun, 32, 64);
        if (FIXED) srun += s2;
        else lse2_merge(mrun, srun, m2, s2);
        if (g == 0 && b < B) m.part[(size_t)b * kMaxSplits + split] = make_float2(mrun, srun);
        __syncthreads();                                      // LDS is reused by the next item
    }
}
#undef RNNLM_A_FRAG

template <int HP>
hipError_t launch_hp(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset, int wg_per_xcd,
                     hipStream_t stream) {
    using C = StagedCfg<HP>;
    static LdsLimit limit[2];
    const void *fn = fixed_offset ? reinterpret_cast<const void *>(outproj_staged_kernel<HP, true>)
                                  : reinterpret_cast<const void *>(outproj_staged_kernel<HP, false>);
    if (hipError_t e = limit[fixed_offset ? 1 : 0].ensure(fn, C::kLdsBytes); e != hipSuccess) return e;
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
    *splits = SplitInfo{0, wg_per_xcd, kStagedRows, kMaxSplits / kXcds, 0};
    switch (m.Hp) {
        case 128: return launch_hp<128>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        case 256: return launch_hp<256>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        case 512: return launch_hp<512>(m, rows, B_dev, fixed_offset, wg_per_xcd, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace rnnlm
