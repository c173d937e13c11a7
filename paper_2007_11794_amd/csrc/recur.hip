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
// scratch block, in the weights' type, as the operand of the output projection.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

__device__ __forceinline__ float sigmoid_f32(float a) {
    // 1/(1+2^(-a log2 e)); the hardware exp2/rcp are accurate to about 1 ulp
    return __frcp_rn(1.0f + fast_exp2(-a * kLog2e));
}

// ----------------------------------------------------------------------------- bf16 / MFMA
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
    // padded units (zero weights, zero embedding) come out as sigmoid(0) - 1/2 = 0
    *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.d) + (size_t)b * Hp + je) = dpk;
    {   // the same four values in the fragment order of the staged output projection
        const size_t frag = (size_t)(b >> 5) * (Hp >> 4) + (je >> 4);
        const size_t at = (frag * 64 + ((je >> 3) & 1) * 32 + (b & 31)) * 8 + (je & 7);
        *reinterpret_cast<uint2 *>(static_cast<bf16_t *>(m.dfrag) + at) = dpk;
    }
    if (vec_ok && je + 4 <= H) {
        *reinterpret_cast<f32x4 *>(h_out + (size_t)bo * H + je) = f32x4{hp[0], hp[1], hp[2], hp[3]};
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (je + i < H) h_out[(size_t)bo * H + je + i] = hp[i];
    }
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
    for (int kb = k_begin; kb < k_end; kb += 8 * kRecurGroups) {
        f32x4 wf[kRecurGroups], hf[kRecurGroups];
#pragma unroll
        for (int u = 0; u < kRecurGroups; ++u) {
            const int k0 = kb + 8 * u;
            if (k0 < k_end) {
                wf[u] = *reinterpret_cast<const f32x4 *>(wrow + k0);
                hf[u] = row_ok ? load4_row(hrow, k0, H, vec_ok, 0.5f) : f32x4{0.5f, 0.5f, 0.5f, 0.5f};
            }
        }
#pragma unroll
        for (int u = 0; u < kRecurGroups; ++u) {
            const int k0 = kb + 8 * u;
            if (k0 < k_end) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(wf[u][e], hf[u][e] - 0.5f, acc, 0, 0, 0);
            }
        }
    }
    const bool w_ok = (w >= 0 && w < m.V);
    const f32x4 u4 = *reinterpret_cast<const f32x4 *>(U + (size_t)(w_ok ? w : 0) * Hp + je);
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
    if (m.dtype == RNNLM_BF16) {
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
