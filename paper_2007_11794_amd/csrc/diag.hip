// Measurement aid, not part of the method: what the bf16 matrix cores of THIS device sustain on a
// loop shaped like the output projection's (Section 2's whole-vocabulary normalisation is where the
// time goes), so that the kernel's rate can be set against what the hardware gives and not only
// against the data-sheet peak.
//
// One workgroup of eight waves per compute unit, as in the staged output projection; every wave
// issues chains of 32 dependent MFMA 32x32x16 (one block of 32 words x 32 rows x 512 units) and
// nothing it does depends on memory after the prologue:
//   feed 0: both operands stay in registers (the bare issue rate of the matrix pipeline);
//   feed 1: the A operand is read from LDS four steps ahead, with the staged kernel's swizzle, and
//           the previous block's 16 logits per lane go through one exp2 and one add each between
//           the MFMAs -- the steady state of the kernel without its loads, barriers and epilogue.
// data 0: all operands zero; data 1: random bf16 of the magnitude of weights and centred
// activations.  The difference between the two is the power-managed clock: the kernel reports
// its core cycles against the constant 100 MHz counter.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "device_utils.h"
#include "rnnlm_diag.h"

namespace rnnlm {

namespace {

constexpr int kProbeThreads = 512;
constexpr int kProbeWorkgroups = 256;
constexpr int kProbeLdsBytes = 128 * 1024;      // as much as keeps a second workgroup off the compute unit
constexpr int kProbeOperands = 4096;            // bf16x8 operands in the input buffer (64 KB)
constexpr int kProbeBlocks = 32;                // chains per wave and launch

template <int FEED>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(const bf16x8 *__restrict__ in,
                                                                   float *__restrict__ out, int blocks,
                                                                   long long *__restrict__ clocks) {
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, col = lane & 31, g = lane >> 5;
    const long long c0 = clock64(), w0 = wall_clock64();
    bf16x8 breg[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) breg[i] = in[(tid + i * kProbeThreads) & (kProbeOperands - 1)];
    // one stage of 32 words x 512 units (32 KB), rows of 1 KB, 16-byte pieces swizzled by the row
    for (int i = tid; i < 2048; i += kProbeThreads)
        *reinterpret_cast<bf16x8 *>(lds + i * 16) = in[i & (kProbeOperands - 1)];
    __syncthreads();
    int aoff[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) aoff[j] = col * 1024 + ((((2 * j) | g) ^ (col & 15)) * 16);
    f32x16 prev;
#pragma unroll
    for (int i = 0; i < 16; ++i) prev[i] = -1.0f * i;
    float srun = 0.f;
    bf16x8 a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) a[i] = *reinterpret_cast<const bf16x8 *>(lds + aoff[i]);
    for (int b = 0; b < blocks; ++b) {
        f32x16 acc = {0};
#pragma unroll
        for (int ks = 0; ks < 32; ++ks) {
            bf16x8 A;
            if (FEED == 1) {
                A = a[ks % 4];
                const int nk = (ks + 4) & 31;            // k-step nk: piece pair nk % 8 of quarter row nk / 8
                a[ks % 4] = *reinterpret_cast<const bf16x8 *>(lds + aoff[nk & 7] + (nk >> 3) * 256);
            } else {
                A = breg[(ks + 7) & 31];
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, breg[ks], acc, 0, 0, 0);
            if (FEED == 1 && (ks & 1)) srun += fast_exp2(prev[ks >> 1] * 1.44269504f + 0.25f);
            __builtin_amdgcn_sched_barrier(0);
        }
        prev = acc;
    }
    float s = srun;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += prev[i];
    out[blockIdx.x * kProbeThreads + tid] = s;            // keeps the work alive
    if (tid == 0 && blockIdx.x == 0) {
        clocks[0] = clock64() - c0;
        clocks[1] = wall_clock64() - w0;
    }
}

struct ProbeBuffers {
    void *in = nullptr, *out = nullptr, *clocks = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    ~ProbeBuffers() {
        (void)hipFree(in);
        (void)hipFree(out);
        (void)hipFree(clocks);
        if (e0) (void)hipEventDestroy(e0);
        if (e1) (void)hipEventDestroy(e1);
    }
};

}  // namespace

}  // namespace rnnlm

using namespace rnnlm;

namespace {
__global__ void empty_kernel(int *sink) {
    if (sink && threadIdx.x == 12345) *sink = 0;             // never true: the kernel does nothing
}
}  // namespace

extern "C" int rnnlm_time_empty_launch(int repeats, void *hip_stream, float *us_per_launch) {
    if (repeats <= 0 || repeats > 100000 || !us_per_launch) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return RNNLM_EDEVICE;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return RNNLM_EDEVICE; }
    int status = RNNLM_OK;
    float ms = 0.f;
    for (int i = 0; i < 10; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s, nullptr);      // warm-up
    if (hipEventRecord(e0, s) != hipSuccess) status = RNNLM_EDEVICE;
    for (int i = 0; i < repeats && status == RNNLM_OK; ++i) hipLaunchKernelGGL(empty_kernel, dim3(1), dim3(64), 0, s, nullptr);
    if (status == RNNLM_OK && (hipEventRecord(e1, s) != hipSuccess || hipEventSynchronize(e1) != hipSuccess ||
                               hipGetLastError() != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess))
        status = RNNLM_EDEVICE;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (status == RNNLM_OK) *us_per_launch = ms * 1e3f / (float)repeats;
    return status;
}

extern "C" int rnnlm_probe_mfma_rate(int feed, int data, int launches, double *tflops, double *core_ghz) {
    if ((feed != 0 && feed != 1) || (data != 0 && data != 1) || launches <= 0 || launches > 1000 || !tflops)
        return RNNLM_EINVAL;
    ProbeBuffers b;
    if (hipMalloc(&b.in, kProbeOperands * sizeof(bf16x8)) != hipSuccess) return RNNLM_ENOMEM;
    if (hipMalloc(&b.out, (size_t)kProbeWorkgroups * kProbeThreads * sizeof(float)) != hipSuccess) return RNNLM_ENOMEM;
    if (hipMalloc(&b.clocks, 2 * sizeof(long long)) != hipSuccess) return RNNLM_ENOMEM;
    if (hipEventCreate(&b.e0) != hipSuccess || hipEventCreate(&b.e1) != hipSuccess) return RNNLM_EDEVICE;
    {
        // random: uniform in +-0.3 and +-0.06 in alternating groups of eight (activations, weights)
        std::vector<uint16_t> h((size_t)kProbeOperands * 8, 0);
        if (data == 1) {
            uint32_t x = 12345u;
            for (size_t i = 0; i < h.size(); ++i) {
                x = x * 1664525u + 1013904223u;
                const float f = ((int)((x >> 8) % 2000u) - 1000) / 1000.0f * ((i & 8) ? 0.06f : 0.3f);
                uint32_t u;
                memcpy(&u, &f, 4);
                h[i] = (uint16_t)(u >> 16);
            }
        }
        if (hipMemcpy(b.in, h.data(), h.size() * 2, hipMemcpyHostToDevice) != hipSuccess) return RNNLM_EDEVICE;
    }
    const void *fn = feed == 1 ? reinterpret_cast<const void *>(mfma_probe_kernel<1>)
                               : reinterpret_cast<const void *>(mfma_probe_kernel<0>);
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, kProbeLdsBytes) != hipSuccess)
        return RNNLM_EDEVICE;
    auto launch = [&]() {
        if (feed == 1)
            hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(kProbeWorkgroups), dim3(kProbeThreads), kProbeLdsBytes, 0,
                               static_cast<const bf16x8 *>(b.in), static_cast<float *>(b.out), kProbeBlocks,
                               static_cast<long long *>(b.clocks));
        else
            hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(kProbeWorkgroups), dim3(kProbeThreads), kProbeLdsBytes, 0,
                               static_cast<const bf16x8 *>(b.in), static_cast<float *>(b.out), kProbeBlocks,
                               static_cast<long long *>(b.clocks));
    };
    launch();                                              // warm-up
    if (hipDeviceSynchronize() != hipSuccess) return RNNLM_EDEVICE;
    if (hipEventRecord(b.e0, 0) != hipSuccess) return RNNLM_EDEVICE;
    for (int i = 0; i < launches; ++i) launch();
    if (hipEventRecord(b.e1, 0) != hipSuccess) return RNNLM_EDEVICE;
    if (hipEventSynchronize(b.e1) != hipSuccess || hipGetLastError() != hipSuccess) return RNNLM_EDEVICE;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, b.e0, b.e1) != hipSuccess || ms <= 0.f) return RNNLM_EDEVICE;
    // 32 x 32 x 16 multiply-adds per MFMA = 32768 flop
    const double flop = (double)launches * kProbeWorkgroups * (kProbeThreads / 64) * kProbeBlocks * 32.0 * 32768.0;
    *tflops = flop / (ms * 1e-3) / 1e12;
    if (core_ghz) {
        long long c[2] = {0, 0};
        if (hipMemcpy(c, b.clocks, sizeof(c), hipMemcpyDeviceToHost) != hipSuccess) return RNNLM_EDEVICE;
        *core_ghz = c[1] > 0 ? (double)c[0] / ((double)c[1] * 10.0) : 0.0;     // wall counter: 100 MHz
    }
    return RNNLM_OK;
}
