// Query gather: only the log-probabilities the search asked for leave the device
// (the paper's aim of exchanging as little as possible, Section 3.2; the returned value is
// the p of Table 1 step 6):
//     logprob[n][k] = z[r][q] - lse[r] (- base_score[n][k], the difference the last paragraph
//     of Section 4.2 sends back),  r = row_of_query[n],  q = query_word[n][k],
// with z[r][q] = bias[q] + sum_j O[j][q] h'[r][j] recomputed as one H-long dot product per
// queried word from the fp32 h' and the [V][H] copy of O (one contiguous row per word), and
// lse[r] assembled from the per-split (max, sum) partials of the output projection in a
// fixed order.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kQueryBatch = 8;

template <typename T>
__global__ __launch_bounds__(256) void query_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int N, int K, SplitInfo si,
    const int32_t *__restrict__ query_word, const int32_t *__restrict__ row_of_query,
    const float *__restrict__ h_out, const float *__restrict__ lse_rows,
    const float *__restrict__ base_score, float *__restrict__ logprob) {
    const int B = B_dev ? *B_dev : rows;
    const int n = blockIdx.x;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int H = m.H, Hp = m.Hp;
    const int r = row_of_query ? row_of_query[n] : n;
    float *out = logprob + (size_t)n * K;
    if (r < 0 || r >= B) {
        if (threadIdx.x == 0) atomicOr(m.flag, RNNLM_FLAG_BAD_ROW);
        for (int k = threadIdx.x; k < K; k += 256) out[k] = quiet_nan();
        return;
    }
    // lse of row r: handed in, or assembled by every wave from the partials, lane l taking
    // splits l, l+64, ...
    float lse;
    if (lse_rows) {
        lse = lse_rows[r];
    } else {
        const int splits = si.fixed_splits > 0 ? si.fixed_splits : staged_plan(B, si.staged_wg_per_xcd).S;
        lse = lse_from_partials(m.part + (size_t)r * kMaxSplits, splits, lane);
    }

    const T *Ot = static_cast<const T *>(m.Ot);
    const float *hrow = h_out + (size_t)r * H;
    const bool vec_ok = (H % 4) == 0;
    // A wave answers the queries k = wave, wave + 4, ...; kQueryBatch of them at a time so
    // that their weight rows are all requested before the first is used.
    for (int kb = wave; kb < K; kb += 4 * kQueryBatch) {
        int q[kQueryBatch];
        bool ok[kQueryBatch];
#pragma unroll
        for (int u = 0; u < kQueryBatch; ++u) {
            const int k = kb + 4 * u;
            q[u] = (k < K) ? query_word[(size_t)n * K + k] : 0;
            ok[u] = (k < K) && q[u] >= 0 && q[u] < m.V;
        }
        float acc[kQueryBatch];
#pragma unroll
        for (int u = 0; u < kQueryBatch; ++u) acc[u] = 0.f;
        for (int j0 = lane * 8; j0 < Hp; j0 += 512) {
            float h8[8];
            load8_row(hrow, j0, H, vec_ok, 0.f, h8);
            float w8[kQueryBatch][8];
#pragma unroll
            for (int u = 0; u < kQueryBatch; ++u) load8_weights(Ot, (size_t)(ok[u] ? q[u] : 0) * Hp + j0, w8[u]);
#pragma unroll
            for (int u = 0; u < kQueryBatch; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u] = fmaf(w8[u][i], h8[i], acc[u]);
        }
#pragma unroll
        for (int u = 0; u < kQueryBatch; ++u) {
            const int k = kb + 4 * u;
            if (k >= K) continue;                        // wave-uniform
            const float z = wave_sum(acc[u]);
            if (lane == 0) {
                if (ok[u]) {
                    const float lp = (z + m.bias[q[u]]) - lse;
                    out[k] = base_score ? lp - base_score[(size_t)n * K + k] : lp;
                }
                else { atomicOr(m.flag, RNNLM_FLAG_BAD_QUERY_WORD); out[k] = quiet_nan(); }
            }
        }
    }
}

}  // namespace

hipError_t launch_query(const ModelDev &m, int rows, const int *B_dev, int N, int K, SplitInfo splits,
                        const int32_t *query_word, const int32_t *row_of_query,
                        const float *h_out, const float *lse_rows, const float *base_score,
                        float *logprob, hipStream_t stream) {
    if (N <= 0 || K <= 0) return hipSuccess;
    if (m.dtype == RNNLM_BF16)
        hipLaunchKernelGGL(query_kernel<bf16_t>, dim3(N), dim3(256), 0, stream, m, rows, B_dev, N, K, splits,
                           query_word, row_of_query, h_out, lse_rows, base_score, logprob);
    else
        hipLaunchKernelGGL(query_kernel<float>, dim3(N), dim3(256), 0, stream, m, rows, B_dev, N, K, splits,
                           query_word, row_of_query, h_out, lse_rows, base_score, logprob);
    return hipGetLastError();
}

}  // namespace rnnlm
