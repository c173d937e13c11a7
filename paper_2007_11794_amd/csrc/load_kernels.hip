// Load-time kernels: re-lay the output weights out as [V][H] (one contiguous row per word:
// the K-major operand of the matrix cores and a single contiguous read per queried word),
// and the per-word constants of the centred logit  z = (bias + colsum(O)/2) + O^T (h' - 1/2).
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

template <typename T>
__global__ __launch_bounds__(256) void transpose_kernel(const T *__restrict__ O, T *__restrict__ Ot,
                                                        int H, int V, int Hp, int Vp) {
    __shared__ T tile[32][33];
    const int v0 = blockIdx.x * 32, j0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        int j = j0 + r, v = v0 + tx;
        tile[r][tx] = (j < H && v < V) ? O[(size_t)j * V + v] : T(0);
    }
    __syncthreads();
    for (int r = ty; r < 32; r += 8) {
        int v = v0 + r, j = j0 + tx;
        if (v < Vp && j < Hp) Ot[(size_t)v * Hp + j] = tile[tx][r];
    }
}

__device__ __forceinline__ double widen(float x) { return (double)x; }
__device__ __forceinline__ double widen(bf16_t x) { return (double)bf16_to_f32(x); }

// Per word v: half the column sum of O, and bounds on the logit that hold for every hidden
// vector with components in [0,1]:  upper = bias + sum_j max(O[j][v],0),
// lower = bias + sum_j min(O[j][v],0).  fp64 accumulation; upper is rounded up and lower
// down by one float ulp-ish margin on the host.
template <typename T>
__global__ __launch_bounds__(256) void col_stats_kernel(const T *__restrict__ O,
                                                        const float *__restrict__ bias, int H, int V,
                                                        float *__restrict__ half_colsum,
                                                        float *__restrict__ upper,
                                                        float *__restrict__ lower) {
    int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= V) return;
    double pos = 0.0, neg = 0.0;
    for (int j = 0; j < H; ++j) {
        double x = widen(O[(size_t)j * V + v]);
        if (x > 0) pos += x; else neg += x;
    }
    double b = bias ? (double)bias[v] : 0.0;
    half_colsum[v] = (float)(0.5 * (pos + neg));
    upper[v] = (float)(b + pos);
    lower[v] = (float)(b + neg);
}

__global__ __launch_bounds__(256) void fill_cvec_kernel(const float *__restrict__ bias,
                                                        const float *__restrict__ half_colsum, int V,
                                                        int Vp, float m2_fixed, float *__restrict__ bias_out,
                                                        float *__restrict__ cvec,
                                                        float *__restrict__ cvec_fixed) {
    int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= Vp) return;
    if (v < V) {
        float b = bias ? bias[v] : 0.f;
        bias_out[v] = b;
        float c = (b + half_colsum[v]) * kLog2e;
        cvec[v] = c;
        cvec_fixed[v] = c - m2_fixed;
    } else {
        cvec[v] = -INFINITY;
        cvec_fixed[v] = -INFINITY;
    }
}

// Three-way bf16 split of the fp32 [Vp][Hp] weights, term-interleaved in chunks of 32 units:
// Ot3[v][j / 32][term][j % 32].
__global__ __launch_bounds__(256) void split3_weights_kernel(const float *__restrict__ Ot, size_t n, int Hp,
                                                             bf16_t *__restrict__ Ot3) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const size_t v = i / Hp;
    const int j = (int)(i % Hp);
    uint16_t t[3];
    split3_bf16(Ot[i], t[0], t[1], t[2]);
    bf16_t *dst = Ot3 + v * 3 * Hp + (size_t)(j >> 5) * 96 + (j & 31);
#pragma unroll
    for (int s = 0; s < 3; ++s) dst[s * 32] = t[s];
}

// bf16 [Vp][Hp] weights re-laid in MFMA-operand order: 16 bytes per thread.
__global__ __launch_bounds__(256) void frag_weights_kernel(const u32x4 *__restrict__ Ot, size_t n, int KS,
                                                           u32x4 *__restrict__ Ofrag) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;       // (blk, ks, lane)
    if (i >= n) return;
    const int lane = (int)(i & 63);
    const size_t frag = i >> 6, blk = frag / KS;
    const int ks = (int)(frag % KS);
    const size_t word = blk * 32 + (lane & 31);
    Ofrag[i] = Ot[word * (2 * KS) + 2 * ks + (lane >> 5)];           // 2 KS chunks of 8 units per word
}

// fp32 [Vp][Hp] weights in the same operand order, 32 bytes per lane as two 16-byte halves:
// [blk][ks][half][64 lanes][4 floats], lane 32 g + c: word 32 blk + c, units 16 ks + 8 g + 4 half .. + 3.
__global__ __launch_bounds__(256) void frag_weights_f32_kernel(const u32x4 *__restrict__ Ot, size_t n, int KS,
                                                               u32x4 *__restrict__ Ofrag) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;       // (blk, ks, half, lane)
    if (i >= n) return;
    const int lane = (int)(i & 63), half = (int)((i >> 6) & 1);
    const size_t frag = i >> 7, blk = frag / KS;
    const int ks = (int)(frag % KS);
    const size_t word = blk * 32 + (lane & 31);
    Ofrag[i] = Ot[word * (4 * KS) + 4 * ks + 2 * (lane >> 5) + half];   // 4 KS chunks of 4 units per word
}

}  // namespace

hipError_t launch_frag_weights(const void *Ot, int dtype, int Vp, int Hp, void *Ofrag, hipStream_t stream) {
    if (dtype == RNNLM_BF16) {
        const size_t n = (size_t)Vp * Hp / 8;
        hipLaunchKernelGGL(frag_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                           static_cast<const u32x4 *>(Ot), n, Hp / 16, static_cast<u32x4 *>(Ofrag));
    } else {
        const size_t n = (size_t)Vp * Hp / 4;
        hipLaunchKernelGGL(frag_weights_f32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                           static_cast<const u32x4 *>(Ot), n, Hp / 16, static_cast<u32x4 *>(Ofrag));
    }
    return hipGetLastError();
}

hipError_t launch_split3_weights(const float *Ot, int Vp, int Hp, void *Ot3, hipStream_t stream) {
    const size_t n = (size_t)Vp * Hp;
    hipLaunchKernelGGL(split3_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, Ot, n, Hp,
                       static_cast<bf16_t *>(Ot3));
    return hipGetLastError();
}

hipError_t launch_transpose_O(const void *O_dev, void *Ot, int dtype, int H, int V, int Hp, int Vp,
                              hipStream_t stream) {
    dim3 grid((Vp + 31) / 32, (Hp + 31) / 32);
    if (dtype == RNNLM_BF16)
        hipLaunchKernelGGL(transpose_kernel<bf16_t>, grid, dim3(256), 0, stream,
                           static_cast<const bf16_t *>(O_dev), static_cast<bf16_t *>(Ot), H, V, Hp, Vp);
    else
        hipLaunchKernelGGL(transpose_kernel<float>, grid, dim3(256), 0, stream,
                           static_cast<const float *>(O_dev), static_cast<float *>(Ot), H, V, Hp, Vp);
    return hipGetLastError();
}

hipError_t launch_col_stats(const void *O_dev, const float *bias, int dtype, int H, int V,
                            float *half_colsum, float *upper, float *lower, hipStream_t stream) {
    dim3 grid((V + 255) / 256);
    if (dtype == RNNLM_BF16)
        hipLaunchKernelGGL(col_stats_kernel<bf16_t>, grid, dim3(256), 0, stream,
                           static_cast<const bf16_t *>(O_dev), bias, H, V, half_colsum, upper, lower);
    else
        hipLaunchKernelGGL(col_stats_kernel<float>, grid, dim3(256), 0, stream,
                           static_cast<const float *>(O_dev), bias, H, V, half_colsum, upper, lower);
    return hipGetLastError();
}

hipError_t launch_fill_cvec(const float *bias, const float *half_colsum, int V, int Vp, float m2_fixed,
                            float *bias_out, float *cvec, float *cvec_fixed, hipStream_t stream) {
    hipLaunchKernelGGL(fill_cvec_kernel, dim3((Vp + 255) / 256), dim3(256), 0, stream, bias, half_colsum,
                       V, Vp, m2_fixed, bias_out, cvec, cvec_fixed);
    return hipGetLastError();
}

}  // namespace rnnlm
