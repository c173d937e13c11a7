// Hidden update  h'[b][j] = sigmoid(U[prev[b]][j] + sum_i W[j][i] h_in[b][i])
// (the context update inside ComputeRnnlm, Table 1 step 6; Section 4.1: the context is the
// previous hidden layer plus the previous word).
//
// The activation enters the product centred: h_in = 1/2 + d, so
//     W h_in = 1/2 rowsum(W) + W d,
// with the first term precomputed at load time in fp64.  |d| <= 1/2 carries three times
// less rounding error than h_in when it is cut to bf16 for the matrix cores, and the bf16
// path additionally splits d = d_hi + d_lo (two MFMA passes; this product is under one
// percent of the step's flops) so that the hidden vector is accurate to fp32 level.
//
// Besides h_out (fp32, caller's buffer) the kernel leaves d' = h' - 1/2 in the model's
// scratch blocks as the operand of the output projection: row-major in the weights' type;
// for bf16 models also times log2(e) in MFMA-fragment order (staged output projection); for
// fp32 models also as three bf16 terms along a six times longer reduction (see ModelDev).
//
// Three kernels: the LDS-tiled bf16 kernel (the default), the register-direct bf16 kernel it
// replaced (kept for hidden sizes that are not a multiple of 4 or unaligned buffers), and the
// fp32 kernel on the full-precision matrix instruction.
#include <limits.h>

#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

__device__ __forceinline__ float sigmoid_f32(float a) {
    // 1/(1+2^(-a log2 e)); the hardware exp2/rcp are accurate to about 1 ulp
    return __frcp_rn(1.0f + fast_exp2(-a * kLog2e));
}

// ----------------------------------------------------------------------------- bf16 / MFMA, register-direct
// A workgroup of 4 waves computes a 32 (units j) x 32 (rows b) block
// D[j][b] = sum_i W[j][i] d[b][i]; wave w takes the quarter w of the reduction length and
// issues all of its loads before the first MFMA (the kernel is bound by load latency, not
// by bytes or flops), the four partial blocks are added through LDS, and wave w finishes
// the units 8 w .. 8 w + 7 of the block.
// MFMA 32x32x16 operand layout (lane l, g = l / 32):
//   A: 8 consecutive k of row (l % 32), starting at 8 g;   B: same for column (l % 32);
//   D: acc[i] is row 8 (i / 4) + 4 g + i % 4, column l % 32.
constexpr int kRecurUnroll = 8;      // k-steps whose loads are in flight together

__global__ __launch_bounds__(256) void recur_bf16_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_dst, const int32_t *__restrict__ prev_word, const float *__restrict__ h_in,
    float *__restrict__ h_out) {
    const int B = B_dev ? *B_dev : rows;
    const int b0 = blockIdx.y * 32;
    if (b0 >= B) return;
    __shared__ f32x4 red[4][4][64];                  // [source wave][quarter of acc][lane]
    const int j0 = blockIdx.x * 32;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, g = lane >> 5;
    const int H = m.H, Hp = m.Hp;
    const bf16_t *W = static_cast<const bf16_t *>(m.W);
    const bf16_t *U = static_cast<const bf16_t *>(m.U);

    const int b = b0 + col;
    const bool row_ok = b < B;
    const int src = row_ok ? (row_src ? row_src[b] : b) : 0;
    const float *hrow = h_in + (size_t)src * H;
    const bool vec_ok = (H % 4) == 0;
    const bf16_t *wrow = W + (size_t)(j0 + col) * Hp;

    // this lane finishes the four units j = j0 + 8 wave + 4 g .. +3 of row b
    const int je = j0 + 8 * wave + 4 * g;
    const int w = row_ok ? prev_word[src] : 0;          // its embedding row is fetched below,
    const f32x4 rs = *reinterpret_cast<const f32x4 *>(m.half_rowsum_W + je);   // after the operands

    const int kq = Hp / 4;                           // this wave's share of k (a multiple of 16)
    const int k_begin = wave * kq + 8 * g, k_end = (wave + 1) * kq;
    f32x16 acc = {0};
    for (int kb = k_begin; kb < k_end; kb += 16 * kRecurUnroll) {
        bf16x8 wf[kRecurUnroll];
        float h8[kRecurUnroll][8];
#pragma unroll
        for (int u = 0; u < kRecurUnroll; ++u) {
            const int k0 = kb + 16 * u;
            if (k0 < k_end) {
                wf[u] = *reinterpret_cast<const bf16x8 *>(wrow + k0);
                if (row_ok) load8_row(hrow, k0, H, vec_ok, 0.5f, h8[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < kRecurUnroll; ++u) {
            const int k0 = kb + 16 * u;
            if (k0 < k_end) {
                u32x4 hi, lo;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    float d0 = row_ok ? h8[u][2 * i] - 0.5f : 0.f, d1 = row_ok ? h8[u][2 * i + 1] - 0.5f : 0.f;
                    hi[i] = pack_bf16x2(d0, d1);
                    lo[i] = pack_bf16x2(d0 - __uint_as_float(hi[i] << 16), d1 - __uint_as_float(hi[i] & 0xFFFF0000u));
                }
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], __builtin_bit_cast(bf16x8, hi), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[u], __builtin_bit_cast(bf16x8, lo), acc, 0, 0, 0);
            }
        }
    }
    const bool w_ok = (w >= 0 && w < m.V);
    const uint2 u4 = *reinterpret_cast<const uint2 *>(U + (size_t)(w_ok ? w : 0) * Hp + je);
#pragma unroll
    for (int q = 0; q < 4; ++q)
        red[wave][q][lane] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    __syncthreads();
    if (!row_ok) return;
    const int bo = row_dst ? row_dst[b] : b;         // row of h_out; the operand block keeps row b
    f32x4 a4 = red[0][wave][lane];
#pragma unroll
    for (int sw = 1; sw < 4; ++sw) {                 // fixed order: deterministic
        f32x4 t = red[sw][wave][lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) a4[i] += t[i];
    }
    if (!w_ok && g == 0 && wave == 0 && blockIdx.x == 0) atomicOr(m.flag, RNNLM_FLAG_BAD_PREV_WORD);
    const float u[4] = {__uint_as_float(u4.x << 16), __uint_as_float(u4.x & 0xFFFF0000u),
                        __uint_as_float(u4.y << 16), __uint_as_float(u4.y & 0xFFFF0000u)};
    float hp[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) hp[i] = w_ok ? sigmoid_f32(a4[i] + rs[i] + u[i]) : quiet_nan();
    uint2 dpk;
    dpk.x = pack_bf16x2(hp[0] - 0.5f, hp[1] - 0.5f);
    dpk.y = pack_bf16x2(hp[2] - 0.5f, hp[3] - 0.5f);
    // padded units (zero weights, zero embedding) come out as sigmoid(0) - 1/2 = 0; either copy of the
    // block is left out (null pointer) when the kernel that follows does not read it
    if (m.d) *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.d) + (size_t)b * Hp + je) = dpk;
    if (m.dfrag) {   // the same four values in the fragment order of the staged output projection
        const size_t frag = (size_t)(b >> 5) * (Hp >> 4) + (je >> 4);
        const size_t at = (frag * 64 + ((je >> 3) & 1) * 32 + (b & 31)) * 8 + (je & 7);
        uint2 dsc;                                       // times log2(e): base-2 logits come out of the MFMAs
        dsc.x = pack_bf16x2((hp[0] - 0.5f) * kLog2e, (hp[1] - 0.5f) * kLog2e);
        dsc.y = pack_bf16x2((hp[2] - 0.5f) * kLog2e, (hp[3] - 0.5f) * kLog2e);
        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.dfrag) + at) = dsc;
    }
    if (vec_ok && je + 4 <= H) {
        *reinterpret_cast<f32x4 *>(h_out + (size_t)bo * H + je) = f32x4{hp[0], hp[1], hp[2], hp[3]};
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (je + i < H) h_out[(size_t)bo * H + je + i] = hp[i];
    }
}

// ----------------------------------------------------------------------------- bf16 / MFMA, LDS-tiled
// The form used when the rows of h_in can be fetched in 16-byte pieces (H a multiple of 4,
// 16-byte aligned buffer).  A workgroup of 2 x 2 waves computes 64 units x 64 rows; a wave
// owns a 32 x 32 block over the whole reduction length (no cross-wave sum).  The reduction
// length is cut in chunks of 64: 64 rows x 128 bytes of W and 64 rows x 256 bytes of h_in
// (kept as two 128-byte half rows), in a ring of four LDS stages filled by direct global->LDS
// loads, each of which covers whole 128-byte lines: the register-direct kernel above touches
// 32 different lines per load instruction and re-reads every operand 2 x more often from L2.
// LDS rows are 128 bytes; chunk c of row r sits at c ^ ((r >> 1) & 7) (as in the tiled
// output projection).  h_in stays fp32 in LDS and is centred and split into hi + lo bf16 in
// registers right before the two MFMAs of a k-step.
constexpr int kRtTile = 64;                           // units per workgroup (and rows, in the large shape)
constexpr int kRtWBytes = kRtTile * 128;              // W part of a stage
// Two shapes (template parameter TB = rows per workgroup):
//   TB = 64: 2 x 2 waves, each a 32 x 32 block over the whole reduction length.  For grids that
//            give every compute unit several workgroups (2 stages, 48 KB, three per unit).
//   TB = 32: a compute unit pulls these direct-to-LDS loads in at 35-50 GB/s only, so a small
//            problem must be spread over ALL compute units with as few bytes per workgroup as
//            possible: 64 units x 32 rows (64 KB of W + 64 KB of h_in for H = 512, against
//            64 + 128 KB), twice as many workgroups.  The four waves are 2 (unit halves) x 2
//            (halves of every chunk's k-steps); the second pair hands its partial sums over
//            through LDS at the end.  4 stages of 16 KB.
template <int TB> struct RtCfg {
    static constexpr int kHalfBytes = TB * 128;                       // one half row per row
    static constexpr int kStageBytes = kRtWBytes + 2 * kHalfBytes;
    static constexpr int kHLoads = TB * 8 / 256;                      // per thread and half
    static constexpr int kLoads = 2 + 2 * kHLoads;                    // per thread and chunk
};

// SUB = chunks per stage and barrier.  With SUB = 2 (small shape, Hp a multiple of 128) a wave
// pair takes one whole chunk of the two: four k-steps of independent loads and conversions
// between two barriers instead of two, which is what the single wave per SIMD needs to hide
// the LDS and matrix latencies.
template <int NS, int TB, int SUB>
__device__ __forceinline__ void recur_bf16_tiled_body(
    const ModelDev &m, int B, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_dst, const int32_t *__restrict__ prev_word, const float *__restrict__ h_in,
    float *__restrict__ h_out) {
    using C = RtCfg<TB>;
    constexpr bool kSplitK = TB == 32;
    // Workgroup id modulo 8 is the XCD (L2 domain).  Row block rb runs on XCD rb % 8 with all
    // its unit blocks, so h_in (the larger operand) is fetched into one L2 only.
    const int JB = m.Hp / kRtTile;
    const int xcd = blockIdx.x % kXcds, local = blockIdx.x / kXcds;
    const int b0 = (xcd + kXcds * (local / JB)) * TB;
    if (b0 >= B) return;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    __shared__ int srcs[TB];
    const int j0 = (local % JB) * kRtTile;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const int wj = wave & 1, wb = kSplitK ? 0 : wave >> 1, wk = kSplitK ? wave >> 1 : 0;
    const int H = m.H, Hp = m.Hp;
    const bf16_t *W = static_cast<const bf16_t *>(m.W);
    const bf16_t *U = static_cast<const bf16_t *>(m.U);

    if (tid < TB) {                                    // rows beyond B repeat the last one; dropped later
        const int rv = min(b0 + tid, B - 1);
        srcs[tid] = row_src ? row_src[rv] : rv;
    }
    __syncthreads();

    // loader: thread fills the physical 16-byte pieces f = q * 256 + tid of an operand tile
    // (row f / 8, position f % 8) with the logical piece c = position ^ swizzle(row)
    uint32_t woff[2];
    const float *hrow[C::kHLoads];
    int hc[C::kHLoads];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        const int f = q * 256 + tid, r = f >> 3, c = (f & 7) ^ ((r >> 1) & 7);
        woff[q] = (uint32_t)(r * Hp * 2 + c * 16);
    }
#pragma unroll
    for (int q = 0; q < C::kHLoads; ++q) {
        const int f = q * 256 + tid, r = f >> 3, c = (f & 7) ^ ((r >> 1) & 7);
        hrow[q] = h_in + (size_t)srcs[r] * H;
        hc[q] = 4 * c;
    }
    const uint32_t wave_s = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = lds_address(lds);
    auto issue = [&](int sc, int stage) {            // the SUB chunks of stage-chunk sc
#pragma unroll
        for (int sub = 0; sub < SUB; ++sub) {
            const int k0 = (sc * SUB + sub) * 64;
            const uint32_t base = lds0 + (stage * SUB + sub) * C::kStageBytes + wave_s * 1024;
            const bf16_t *wsrc = W + (size_t)j0 * Hp + k0;
#pragma unroll
            for (int q = 0; q < 2; ++q) lds_dma_16(wsrc, woff[q], base + q * 4096);
#pragma unroll
            for (int half = 0; half < 2; ++half)
#pragma unroll
                for (int q = 0; q < C::kHLoads; ++q) {
                    // pieces past the end of the row meet zero weights: fetch the row's first piece
                    const int k = k0 + 32 * half + hc[q];
                    lds_dma_16_ptr(hrow[q] + (k + 4 <= H ? k : 0),
                                   base + kRtWBytes + half * C::kHalfBytes + q * 4096);
                }
        }
    };

    const int b = b0 + 32 * wb + col;
    const bool row_ok = b < B;
    const int src = srcs[32 * wb + col];
    const int w = prev_word[src];
    const bool w_ok = (w >= 0 && w < m.V);
    const int jw = j0 + 32 * wj + 4 * g;                // this lane finishes units jw + 8 q .. + 3, q < 4
    const int nk = Hp / (64 * SUB);                     // stage-chunks (the launcher checks divisibility)
#pragma unroll
    for (int c = 0; c < NS - 1; ++c)
        if (c < nk) issue(c, c);
    uint2 u4[4];
    f32x4 rs[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        u4[q] = *reinterpret_cast<const uint2 *>(U + (size_t)(w_ok ? w : 0) * Hp + jw + 8 * q);
        rs[q] = *reinterpret_cast<const f32x4 *>(m.half_rowsum_W + jw + 8 * q);
    }

    // LDS offsets of this lane's operands at k-step ks of a chunk
    int aoff[4], boff[4];
    {
        const int ra = 32 * wj + col, rb = 32 * wb + col;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            aoff[ks] = ra * 128 + (((2 * ks + g) ^ ((ra >> 1) & 7)) * 16);
            // h: k = 16 ks + 8 g .. + 7 -> half row ks / 2, pieces 4 (ks % 2) + 2 g and the next
            boff[ks] = kRtWBytes + (ks >> 1) * C::kHalfBytes + rb * 128;
        }
    }
    const int bsw = ((32 * wb + col) >> 1) & 7;

    f32x16 acc = {0};
    for (int chunk = 0; chunk < nk; ++chunk) {
        const int stage = chunk % NS;
        // my loads of this chunk have landed once only those of the (at most two) later chunks
        // already requested are outstanding
        const int later = min(NS - 2, nk - 1 - chunk);
        if (later >= 2) wait_vmcnt<2 * SUB * C::kLoads>();
        else if (later == 1) wait_vmcnt<SUB * C::kLoads>();
        else wait_vmcnt<0>();
        __syncthreads();                                // everybody's; the stage of chunk - 1 is free
        if (chunk + NS - 1 < nk) issue(chunk + NS - 1, (chunk + NS - 1) % NS);
        // split reduction: with two chunks per stage a wave pair takes one of them, else half of
        // the k-steps of the one chunk
        const char *st = lds + (stage * SUB + (SUB == 2 ? wk : 0)) * C::kStageBytes;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (kSplitK && SUB == 1 && (ks >> 1) != wk) continue;   // wave-uniform
            const bf16x8 a = *reinterpret_cast<const bf16x8 *>(st + aoff[ks]);
            const int c0 = 4 * (ks & 1) + 2 * g;
            const f32x4 h0 = *reinterpret_cast<const f32x4 *>(st + boff[ks] + ((c0 ^ bsw) * 16));
            const f32x4 h1 = *reinterpret_cast<const f32x4 *>(st + boff[ks] + (((c0 + 1) ^ bsw) * 16));
            const float h8[8] = {h0[0], h0[1], h0[2], h0[3], h1[0], h1[1], h1[2], h1[3]};
            u32x4 hi, lo;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float d0 = h8[2 * i] - 0.5f, d1 = h8[2 * i + 1] - 0.5f;
                hi[i] = pack_bf16x2(d0, d1);
                lo[i] = pack_bf16x2(d0 - __uint_as_float(hi[i] << 16), d1 - __uint_as_float(hi[i] & 0xFFFF0000u));
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, hi), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, __builtin_bit_cast(bf16x8, lo), acc, 0, 0, 0);
        }
    }
    if (kSplitK) {
        // the waves with the second halves hand their sums to their partners (the stages are free now)
        f32x4 *red = reinterpret_cast<f32x4 *>(lds) + (size_t)wj * 4 * 64;
        __syncthreads();
        if (wk == 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q) red[q * 64 + lane] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
        }
        __syncthreads();
        if (wk == 1) return;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const f32x4 t = red[q * 64 + lane];
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[4 * q + i] += t[i];
        }
    }
    if (!row_ok) return;
    if (!w_ok && g == 0 && wj == 0 && j0 == 0) atomicOr(m.flag, RNNLM_FLAG_BAD_PREV_WORD);
    const int bo = row_dst ? row_dst[b] : b;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int je = jw + 8 * q;
        const float u[4] = {__uint_as_float(u4[q].x << 16), __uint_as_float(u4[q].x & 0xFFFF0000u),
                            __uint_as_float(u4[q].y << 16), __uint_as_float(u4[q].y & 0xFFFF0000u)};
        float hp[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) hp[i] = w_ok ? sigmoid_f32(acc[4 * q + i] + rs[q][i] + u[i]) : quiet_nan();
        uint2 dpk;                                      // padded units come out as sigmoid(0) - 1/2 = 0
        dpk.x = pack_bf16x2(hp[0] - 0.5f, hp[1] - 0.5f);
        dpk.y = pack_bf16x2(hp[2] - 0.5f, hp[3] - 0.5f);
        // either copy of the block is left out (null pointer) when the kernel that follows does not read it
        if (m.d) *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.d) + (size_t)b * Hp + je) = dpk;
        if (m.dfrag) {
            const size_t frag = (size_t)(b >> 5) * (Hp >> 4) + (je >> 4);
            const size_t at = (frag * 64 + ((je >> 3) & 1) * 32 + (b & 31)) * 8 + (je & 7);
            uint2 dsc;                                   // times log2(e): base-2 logits come out of the MFMAs
            dsc.x = pack_bf16x2((hp[0] - 0.5f) * kLog2e, (hp[1] - 0.5f) * kLog2e);
            dsc.y = pack_bf16x2((hp[2] - 0.5f) * kLog2e, (hp[3] - 0.5f) * kLog2e);
            *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.dfrag) + at) = dsc;
        }
        if (je + 4 <= H) *reinterpret_cast<f32x4 *>(h_out + (size_t)bo * H + je) = f32x4{hp[0], hp[1], hp[2], hp[3]};
    }
}

template <int NS, int TB, int SUB>
__global__ __launch_bounds__(256) void recur_bf16_tiled_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_dst, const int32_t *__restrict__ prev_word, const float *__restrict__ h_in,
    float *__restrict__ h_out, int b_min, int b_max, int small_upto) {
    // When only the device knows the row count, both shapes are launched and the count picks one:
    // the launch whose range the count is not in sees no rows.  (Folded into B, not a branch of
    // its own: a branch here would put two more dependent scalar loads in front of everything.)
    const int B_true = B_dev ? *B_dev : rows;
    const int B = (B_true < b_min || B_true > b_max) ? 0 : B_true;
    if constexpr (TB == 64) {
        // A launch of the large shape sized for a bound far above the true count (a step most of whose
        // histories were found in the cache) would leave a handful of workgroups with 192 KB each to pull
        // in.  Up to small_upto rows the same workgroups take 32 rows each instead (the small shape's
        // body in this launch's LDS: three stages of 16 KB), twice as many of them at work.
        static_assert(2 * RtCfg<64>::kStageBytes == 3 * RtCfg<32>::kStageBytes, "the small body's stages fit this launch's LDS");
        if (B <= small_upto) {                            // uniform
            recur_bf16_tiled_body<3, 32, 1>(m, B, row_src, row_dst, prev_word, h_in, h_out);
            return;
        }
    }
    recur_bf16_tiled_body<NS, TB, SUB>(m, B, row_src, row_dst, prev_word, h_in, h_out);
}

// ----------------------------------------------------------------------------- fp32 / MFMA
// Same shape as the bf16 kernel (32 x 32 block per workgroup, reduction length split over the
// four waves, all loads of a wave in flight together), with the full-precision fp32 matrix
// instruction 32x32x2: per lane one float of A (row l % 32, k = l / 32) and one of B.  A lane
// loads four consecutive k at a time (lane half g takes k0 + 4 g .. + 3); MFMA number e of the
// group multiplies the k pair {k0 + e, k0 + 4 + e}, the same pairing for both operands.
constexpr int kRecurGroups = 8;      // groups of 8 k whose loads are in flight together

__device__ __forceinline__ f32x4 load4_row(const float *row, int k0, int H, bool vec_ok, float fill) {
    if (vec_ok && k0 + 4 <= H) return *reinterpret_cast<const f32x4 *>(row + k0);
    f32x4 v;
#pragma unroll
    for (int i = 0; i < 4; ++i) v[i] = (k0 + i < H) ? row[k0 + i] : fill;
    return v;
}

__global__ __launch_bounds__(256) void recur_f32_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, const int32_t *__restrict__ row_src,
    const int32_t *__restrict__ row_dst, const int32_t *__restrict__ prev_word, const float *__restrict__ h_in,
    float *__restrict__ h_out) {
    const int B = B_dev ? *B_dev : rows;
    const int b0 = blockIdx.y * 32;
    if (b0 >= B) return;
    __shared__ f32x4 red[4][4][64];                  // [source wave][quarter of acc][lane]
    const int j0 = blockIdx.x * 32;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, col = lane & 31, g = lane >> 5;
    const int H = m.H, Hp = m.Hp;
    const float *W = static_cast<const float *>(m.W);
    const float *U = static_cast<const float *>(m.U);

    const int b = b0 + col;
    const bool row_ok = b < B;
    const int src = row_ok ? (row_src ? row_src[b] : b) : 0;
    const float *hrow = h_in + (size_t)src * H;
    const bool vec_ok = (H % 4) == 0;
    const float *wrow = W + (size_t)(j0 + col) * Hp;
    const int je = j0 + 8 * wave + 4 * g;            // the four units this lane finishes
    const int w = row_ok ? prev_word[src] : 0;
    const f32x4 rs = *reinterpret_cast<const f32x4 *>(m.half_rowsum_W + je);

    const int kq = Hp / 4;                           // this wave's share of k (a multiple of 16)
    const int k_begin = wave * kq + 4 * g, k_end = (wave + 1) * kq;
    f32x16 acc = {0};
    f32x4 wf[kRecurGroups], hf[kRecurGroups];
    auto request = [&](int kb) {
#pragma unroll
        for (int u = 0; u < kRecurGroups; ++u) {
            const int k0 = kb + 8 * u;
            if (k0 < k_end) {
                wf[u] = *reinterpret_cast<const f32x4 *>(wrow + k0);
                hf[u] = row_ok ? load4_row(hrow, k0, H, vec_ok, 0.5f) : f32x4{0.5f, 0.5f, 0.5f, 0.5f};
            }
        }
    };
    auto multiply = [&](int kb) {
#pragma unroll
        for (int u = 0; u < kRecurGroups; ++u) {
            const int k0 = kb + 8 * u;
            if (k0 < k_end) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[u][e], hf[u][e] - 0.5f, acc, 0, 0, 0);
            }
        }
    };
    // The embedding row hangs on the previous word, one round trip behind the operands of the first
    // groups: requested right after them, it is on its way while the matrix instructions run.
    request(k_begin);
    const bool w_ok = (w >= 0 && w < m.V);
    const f32x4 u4 = *reinterpret_cast<const f32x4 *>(U + (size_t)(w_ok ? w : 0) * Hp + je);
    multiply(k_begin);
    for (int kb = k_begin + 8 * kRecurGroups; kb < k_end; kb += 8 * kRecurGroups) {
        request(kb);
        multiply(kb);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
        red[wave][q][lane] = f32x4{acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]};
    __syncthreads();
    if (!row_ok) return;
    const int bo = row_dst ? row_dst[b] : b;         // row of h_out; the operand block keeps row b
    f32x4 a4 = red[0][wave][lane];
#pragma unroll
    for (int sw = 1; sw < 4; ++sw) {                 // fixed order: deterministic
        f32x4 t = red[sw][wave][lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) a4[i] += t[i];
    }
    if (!w_ok && g == 0 && wave == 0 && blockIdx.x == 0) atomicOr(m.flag, RNNLM_FLAG_BAD_PREV_WORD);
    f32x4 hp, dv;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        hp[i] = w_ok ? sigmoid_f32(a4[i] + rs[i] + u4[i]) : quiet_nan();
        dv[i] = hp[i] - 0.5f;                        // padded units: sigmoid(0) - 1/2 = 0
    }
    *reinterpret_cast<f32x4 *>(static_cast<float *>(m.d) + (size_t)b * Hp + je) = dv;
    if (m.d3) {     // the same values as three bf16 terms, term-interleaved in chunks of 32 units
        uint16_t t[4][3];
#pragma unroll
        for (int i = 0; i < 4; ++i) split3_bf16(dv[i], t[i][0], t[i][1], t[i][2]);
        bf16_t *row3 = static_cast<bf16_t *>(m.d3) + (size_t)b * 3 * Hp + (size_t)(je >> 5) * 96 + (je & 31);
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            uint2 pk;
            pk.x = (uint32_t)t[0][k] | ((uint32_t)t[1][k] << 16);
            pk.y = (uint32_t)t[2][k] | ((uint32_t)t[3][k] << 16);
            *reinterpret_cast<uint2 *>(row3 + k * 32) = pk;
        }
    }
    if (vec_ok && je + 4 <= H) {
        *reinterpret_cast<f32x4 *>(h_out + (size_t)bo * H + je) = hp;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (je + i < H) h_out[(size_t)bo * H + je + i] = hp[i];
    }
}

}  // namespace

hipError_t launch_recur(const ModelDev &m, int rows, const int *B_dev, const int32_t *row_src,
                        const int32_t *row_dst, const int32_t *prev_word, const float *h_in,
                        float *h_out, hipStream_t stream) {
    if (rows <= 0) return hipSuccess;
    if (m.dtype == RNNLM_BF16 && m.H % 4 == 0 && (reinterpret_cast<uintptr_t>(h_in) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(h_out) & 15) == 0) {
        const int units = m.Hp / kRtTile;
        static LdsLimit limit[2];                       // the small shape takes more than the default 64 KB of dynamic LDS
        if (hipError_t e = limit[0].ensure(reinterpret_cast<const void *>(recur_bf16_tiled_kernel<4, 32, 1>),
                                           4 * RtCfg<32>::kStageBytes);
            e != hipSuccess)
            return e;
        if (hipError_t e = limit[1].ensure(reinterpret_cast<const void *>(recur_bf16_tiled_kernel<4, 32, 2>),
                                           8 * RtCfg<32>::kStageBytes);
            e != hipSuccess)
            return e;
        // The small shape (32 rows per workgroup) while its workgroups fit the compute units in one
        // round, the large one (64 rows, three workgroups per unit) beyond: the crossover measured
        // at H = 512, 768, 1024 and 2048 lies there.
        const int small_max = 32 * (256 / units);       // most rows the small shape is chosen for
        auto launch_big = [&](int b_min) {
            const int big_blocks = (rows + 63) / 64;
            const int slots = kXcds * ((big_blocks + kXcds - 1) / kXcds);   // row blocks the grid has workgroups for
            dim3 grid(slots * units);
            // true counts up to here are served 32 rows per workgroup (see the kernel)
            const int small_upto = B_dev ? std::min(small_max, 32 * slots) : 0;
            hipLaunchKernelGGL((recur_bf16_tiled_kernel<2, 64, 1>), grid, dim3(256), 2 * RtCfg<64>::kStageBytes, stream,
                               m, rows, B_dev, row_src, row_dst, prev_word, h_in, h_out, b_min, INT_MAX, small_upto);
        };
        auto launch_small = [&](int upto) {             // grid for `upto` rows
            const int small_blocks = (upto + 31) / 32;
            dim3 grid(kXcds * ((small_blocks + kXcds - 1) / kXcds) * units);
            if (m.Hp % 128 == 0)
                hipLaunchKernelGGL((recur_bf16_tiled_kernel<4, 32, 2>), grid, dim3(256), 8 * RtCfg<32>::kStageBytes,
                                   stream, m, rows, B_dev, row_src, row_dst, prev_word, h_in, h_out, 0, upto, 0);
            else
                hipLaunchKernelGGL((recur_bf16_tiled_kernel<4, 32, 1>), grid, dim3(256), 4 * RtCfg<32>::kStageBytes,
                                   stream, m, rows, B_dev, row_src, row_dst, prev_word, h_in, h_out, 0, upto, 0);
        };
        if (rows <= small_max) {
            launch_small(rows);
        } else if (B_dev && small_max > 0 && m.Hp >= 1024) {
            // The true count may be far below the bound: launch both, the count on the device picks
            // and the other one ends at once.  The extra launch costs 1 to 3 us per step; for few rows
            // the small shape saves 5 us from Hp = 1024 on and under 1 us at Hp = 768 (measured).
            launch_small(small_max);
            launch_big(small_max + 1);
        } else {
            launch_big(0);
        }
    } else if (m.dtype == RNNLM_BF16) {
        dim3 grid(m.Hp / 32, (rows + 31) / 32);
        hipLaunchKernelGGL(recur_bf16_kernel, grid, dim3(256), 0, stream, m, rows, B_dev, row_src,
                           row_dst, prev_word, h_in, h_out);
    } else {
        dim3 grid(m.Hp / 32, (rows + 31) / 32);
        hipLaunchKernelGGL(recur_f32_kernel, grid, dim3(256), 0, stream, m, rows, B_dev, row_src,
                           row_dst, prev_word, h_in, h_out);
    }
    return hipGetLastError();
}

}  // namespace rnnlm
