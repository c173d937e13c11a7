// Output projection + log-sum-exp for FEW rows: the weight-streaming kernels (bf16 models first,
// fp32 models at the end of the file).
//
// What is computed is the same as in the other output-projection kernels (normalising over
// all words of the vocabulary, Section 2.1 of the paper).  With a handful of distinct
// histories in a step -- the paper's search re-asks the same context most of the time
// (Section 5.2), so few rows are left after the lookup -- the contraction is a thin one:
// every weight is used for at most a few dozen rows, and the time is the time to read the
// output weights once.  So this kernel is built around the memory system, not the matrix core:
//   - the weights are read from a second copy kept in MFMA-operand order (Ofrag: one operand
//     of a wave = 32 words x 16 units = 1 KB contiguous), so every load instruction of a wave
//     is one fully coalesced kilobyte straight into the registers the MFMA reads: no LDS
//     round trip, no barrier, no partial cache lines;
//   - a wave owns whole 32-word blocks and keeps a ring of kStreamRing groups of kGroup operands in
//     flight (16 KB per wave, 128 KB per CU with 8 waves, 32 MB over the chip: more than
//     bandwidth x latency of HBM), waves never synchronise inside the loop;
//   - the hidden block (<= 32 RB rows, times log2 e, already in operand order) sits in LDS and is
//     read per MFMA; one weight operand feeds RB MFMAs;
//   - exp-and-add per block in registers as elsewhere; at the end the eight waves' (max, sum)
//     pairs are merged through LDS in a fixed order: one partial per row and workgroup.
#include "device_utils.h"
#include "outproj_stream_body.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kThreads = kStreamThreads;
typedef StreamCursor Cursor;

template <int RB, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_stream_kernel(ModelDev m, int rows,
                                                                  const int *__restrict__ B_dev, int row0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // this launch serves rows row0 .. row0 + 32 RB - 1 (row0 a multiple of 32)
    const int B = (B_dev ? *B_dev : rows) - row0;
    if (B <= 0) return;                                       // uniform: no barrier is met
    outproj_stream_body<RB, FIXED>(m, B, row0, blockIdx.x, gridDim.x, lds);
}

// ------------------------------------------------------------------------------ fp32 models
template <int RB, bool FIXED>
__global__ __launch_bounds__(kThreads) void outproj_stream_f32_kernel(ModelDev m, int rows,
                                                                      const int *__restrict__ B_dev, int row0) {
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int B = (B_dev ? *B_dev : rows) - row0;
    if (B <= 0) return;                                       // uniform: no barrier is met
    outproj_stream_f32_body<RB, FIXED>(m, B, row0, blockIdx.x, gridDim.x, lds);
}

template <int RB>
hipError_t launch_rb(const ModelDev &m, int rows, const int *B_dev, int row0, bool fixed_offset, int S,
                     hipStream_t stream) {
    static LdsLimit limit[4];
    const bool f32 = m.dtype == RNNLM_F32;
    const int which = (fixed_offset ? 1 : 0) + (f32 ? 2 : 0);
    const size_t lds_bytes = stream_lds_bytes(f32 ? 3 : 1, RB, m.Hp >> 4);
    const void *fn = f32 ? (fixed_offset ? reinterpret_cast<const void *>(outproj_stream_f32_kernel<RB, true>)
                                         : reinterpret_cast<const void *>(outproj_stream_f32_kernel<RB, false>))
                         : (fixed_offset ? reinterpret_cast<const void *>(outproj_stream_kernel<RB, true>)
                                         : reinterpret_cast<const void *>(outproj_stream_kernel<RB, false>));
    if (hipError_t e = limit[which].ensure(fn, lds_bytes); e != hipSuccess) return e;
    if (f32) {
        if (fixed_offset)
            hipLaunchKernelGGL((outproj_stream_f32_kernel<RB, true>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
        else
            hipLaunchKernelGGL((outproj_stream_f32_kernel<RB, false>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
    } else {
        if (fixed_offset)
            hipLaunchKernelGGL((outproj_stream_kernel<RB, true>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
        else
            hipLaunchKernelGGL((outproj_stream_kernel<RB, false>), dim3(S), dim3(kThreads), lds_bytes, stream, m, rows, B_dev, row0);
    }
    return hipGetLastError();
}

}  // namespace

// Rows the streaming kernel can take for this model: the hidden block (bf16 models: one copy;
// fp32 models: its three bf16 terms) must fit in LDS.
int outproj_stream_max_rows(const ModelDev &m) {
    if (!m.Ofrag || m.hs) return 0;
    if (m.dtype == RNNLM_BF16 && !m.dfrag) return 0;
    const int KS = m.Hp >> 4, terms = m.dtype == RNNLM_F32 ? 3 : 1;
    int rb = 0;
    for (int c = 1; c <= 4; c *= 2)
        if (stream_lds_bytes(terms, c, KS) <= 156 * 1024) rb = c;          // of the 160 KB a workgroup can have
    return 32 * rb;
}

// Rows beyond what one launch holds in LDS are served by further launches (each streams the weights
// again: worth it for a few passes only, the caller decides).
hipError_t launch_outproj_stream(const ModelDev &m, int rows, const int *B_dev, bool fixed_offset,
                                 SplitInfo *splits, hipStream_t stream) {
    const int per = outproj_stream_max_rows(m);
    if (per == 0) return hipErrorInvalidValue;
    const int T = m.Vp / 32;
    const int S = T < kMaxSplits ? T : kMaxSplits;
    *splits = fixed_split_info(S);
    for (int row0 = 0; row0 < rows; row0 += per) {
        const int n = rows - row0 < per ? rows - row0 : per;
        hipError_t e = n <= 32   ? launch_rb<1>(m, rows, B_dev, row0, fixed_offset, S, stream)
                       : n <= 64 ? launch_rb<2>(m, rows, B_dev, row0, fixed_offset, S, stream)
                                 : launch_rb<4>(m, rows, B_dev, row0, fixed_offset, S, stream);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace rnnlm
