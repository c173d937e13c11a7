// Query gather: only the log-probabilities the search asked for leave the device
// (the paper's aim of exchanging as little as possible, Section 3.2; the returned value is
// the p of Table 1 step 6):
//     logprob[n][k] = z[r][q] - lse[r] (- base_score[n][k], the difference the last paragraph
//     of Section 4.2 sends back),  r = row_of_query[n],  q = query_word[n][k],
// with z[r][q] = bias[q] + sum_j O[j][q] h'[r][j] recomputed as one H-long dot product per
// queried word from the fp32 h' and the [V][H] copy of O (one contiguous row per word), and
// lse[r] assembled from the per-split (max, sum) partials of the output projection in a
// fixed order.
//
// Through a cache kept between steps (CACHED) the same kernel also does what Table 1 does after
// ComputeRnnlm: a history found in the cache takes h' and lse from the stores, a computed one from
// this step's block; and the wave that serves the FIRST raw query of a distinct history (rep[u])
// passes the h' it is reading anyway on: to the caller's h_out for a found history, into the
// store (with lse) for a new entry.  No other wave reads what it writes in this launch.
#include "device_utils.h"
#include "rnnlm_internal.h"

namespace rnnlm {

namespace {

constexpr int kQueryBatch = 8;

// A workgroup of four waves serves QPW raw queries (4, 2 or 1): with few words per query a
// whole wave per query keeps the eight-row batches full; with many, the four waves share
// one query's words.  Nothing branches on loaded values before the stores, so the loads of
// a batch (row index, word ids, their bias and base score, the partials, eight weight rows,
// the hidden row) are in flight together.
__device__ __forceinline__ void store8_row(float *row, int k0, int H, bool vec_ok, const float (&v)[8]) {
    if (vec_ok && k0 + 8 <= H) {
        *reinterpret_cast<f32x4 *>(row + k0) = f32x4{v[0], v[1], v[2], v[3]};
        *reinterpret_cast<f32x4 *>(row + k0 + 4) = f32x4{v[4], v[5], v[6], v[7]};
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (k0 + i < H) row[k0 + i] = v[i];
    }
}

template <typename T, int QPW, bool CACHED>
__global__ __launch_bounds__(256) void query_kernel(
    ModelDev m, int rows, const int *__restrict__ B_dev, int N, int K, SplitInfo si,
    const int32_t *__restrict__ query_word, const int32_t *__restrict__ row_of_query,
    float *__restrict__ h_out, const float *__restrict__ lse_rows,
    const float *__restrict__ base_score, float *__restrict__ logprob, CacheDev c,
    const int32_t *__restrict__ rep) {
    constexpr int kWavesPerQuery = 4 / QPW;
    constexpr int kPartsPerLane = kMaxSplits / 64;
    const int B = B_dev ? *B_dev : rows;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int n = blockIdx.x * QPW + wave / kWavesPerQuery;
    if (n >= N) return;                                  // wave-uniform; no barrier in this kernel
    const int kwave = wave % kWavesPerQuery;             // this wave takes words kwave, kwave + 4/QPW, ...
    const int H = m.H, Hp = m.Hp;
    // The word ids of the first batch depend on n only: requested before anything that hangs on the
    // row index, so that the weight rows can follow one memory latency after the start, not three.
    const int umine = batch_slot_of_lane(lane);
    const int k_first = kwave + kWavesPerQuery * umine;
    const int q_first = (k_first < K) ? query_word[(size_t)n * K + k_first] : 0;
    const int r_raw = row_of_query ? row_of_query[n] : n;
    const bool r_ok = r_raw >= 0 && r_raw < B;
    const int r = r_ok ? r_raw : 0;                      // a bad row is computed on row 0 and then dropped
    float *out = logprob + (size_t)n * K;
    const bool writer = (lane & 7) == 0;

    // lse of row r: handed in, or merged from the partials (lane l takes splits l, l+64, ...)
    // once the first batch of dot products is done.
    // through the cache: row of this step's computed block (or -1: found) and entry of history r
    int prow = r, entry = -1;
    if (CACHED) { prow = c.miss_of[r]; entry = c.entry_of[r]; }
    const bool computed = !CACHED || prow >= 0;
    float2 parts[kPartsPerLane];
    float lse = 0.f, stored_lse = 0.f;
    if (lse_rows) {
        lse = lse_rows[r];
    } else {
        // (found histories load the partials of row 0 and never use them: no branch before the loads)
        const int pr = prow > 0 ? prow : 0;
        const int splits = splits_of(si, CACHED ? *c.n_miss : B);
#pragma unroll
        for (int i = 0; i < kPartsPerLane; ++i) {
            const int s = lane + 64 * i;
            const float2 p = m.part[(size_t)pr * kMaxSplits + (s < splits ? s : 0)];
            parts[i] = (s < splits) ? p : make_float2(-INFINITY, 0.f);
        }
        if (CACHED) stored_lse = c.store_lse[entry > 0 ? entry : 0];
    }

    const T *Ot = static_cast<const T *>(m.Ot);
    const float *hrow = computed ? h_out + (size_t)r * H : c.store_h + (size_t)entry * H;
    // the wave that passes h' on (first raw query of the history, first word group), and where to
    float *pass_to = nullptr;
    bool owner = false;
    if (CACHED) {
        owner = r_ok && kwave == 0 && rep[r] == n;
        if (owner) pass_to = computed ? (entry >= 0 ? c.store_h + (size_t)entry * H : nullptr) : h_out + (size_t)r * H;
    }
    const bool vec_ok = (H % 4) == 0;
    for (int kb = kwave; kb < K; kb += kWavesPerQuery * kQueryBatch) {
        // this lane's word of the batch, its bias and base score
        const int kmine = kb + kWavesPerQuery * umine;
        const bool k_ok = kmine < K;
        const int qmine = (kb == kwave) ? q_first : (k_ok ? query_word[(size_t)n * K + kmine] : 0);
        const bool q_ok = qmine >= 0 && qmine < m.V;
        const int qsafe = q_ok ? qmine : 0;
        const float bias_mine = m.bias[qsafe];
        const float base_mine = (base_score && k_ok) ? base_score[(size_t)n * K + kmine] : 0.f;
        int q[kQueryBatch];                              // wave-uniform word ids of the batch
#pragma unroll
        for (int u = 0; u < kQueryBatch; ++u) q[u] = __builtin_amdgcn_readlane(qsafe, lane_of_batch_slot(u));

        float acc[kQueryBatch];
#pragma unroll
        for (int u = 0; u < kQueryBatch; ++u) acc[u] = 0.f;
        for (int j0 = lane * 8; j0 < Hp; j0 += 512) {
            float h8[8];
            load8_row(hrow, j0, H, vec_ok, 0.f, h8);
            if (CACHED && pass_to && kb == kwave) store8_row(pass_to, j0, H, vec_ok, h8);
            float w8[kQueryBatch][8];
#pragma unroll
            for (int u = 0; u < kQueryBatch; ++u) load8_weights(Ot, (size_t)q[u] * Hp + j0, w8[u]);
#pragma unroll
            for (int u = 0; u < kQueryBatch; ++u)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[u] = fmaf(w8[u][i], h8[i], acc[u]);
        }
        if (!lse_rows && kb == kwave) {                  // first batch: merge the partials now
            float pm = -INFINITY, ps = 0.f;
#pragma unroll
            for (int i = 0; i < kPartsPerLane; ++i) lse2_merge(pm, ps, parts[i].x, parts[i].y);
            const float mm = wave_max(pm);
            const float ss = wave_sum(mm == -INFINITY ? 0.f : ps * fast_exp2(pm - mm));
            lse = (mm + fast_log2(ss)) * kLn2;
            if (CACHED) {
                if (!computed) lse = stored_lse;
                else if (owner && entry >= 0 && lane == 0) c.store_lse[entry] = lse;
            }
        }
        const float z = wave_sum8(acc, lane);
        if (writer && k_ok) {
            if (r_ok && q_ok) {
                float lp = (z + bias_mine) - lse;
                if (base_score) lp -= base_mine;
                out[kmine] = lp;
            } else {
                atomicOr(m.flag, r_ok ? RNNLM_FLAG_BAD_QUERY_WORD : RNNLM_FLAG_BAD_ROW);
                out[kmine] = quiet_nan();
            }
        }
    }
}

}  // namespace

namespace {
template <typename T, bool CACHED>
void launch_query_typed(const ModelDev &m, int rows, const int *B_dev, int N, int K, SplitInfo splits,
                        const int32_t *query_word, const int32_t *row_of_query, float *h_out,
                        const float *lse_rows, const float *base_score, float *logprob, const CacheDev &c,
                        const int32_t *rep, hipStream_t stream) {
    if (K <= kQueryBatch)
        hipLaunchKernelGGL((query_kernel<T, 4, CACHED>), dim3((N + 3) / 4), dim3(256), 0, stream, m, rows, B_dev, N,
                           K, splits, query_word, row_of_query, h_out, lse_rows, base_score, logprob, c, rep);
    else if (K <= 2 * kQueryBatch)
        hipLaunchKernelGGL((query_kernel<T, 2, CACHED>), dim3((N + 1) / 2), dim3(256), 0, stream, m, rows, B_dev, N,
                           K, splits, query_word, row_of_query, h_out, lse_rows, base_score, logprob, c, rep);
    else
        hipLaunchKernelGGL((query_kernel<T, 1, CACHED>), dim3(N), dim3(256), 0, stream, m, rows, B_dev, N, K, splits,
                           query_word, row_of_query, h_out, lse_rows, base_score, logprob, c, rep);
}
}  // namespace

hipError_t launch_query(const ModelDev &m, int rows, const int *B_dev, int N, int K, SplitInfo splits,
                        const int32_t *query_word, const int32_t *row_of_query,
                        const float *h_out, const float *lse_rows, const float *base_score,
                        float *logprob, hipStream_t stream) {
    if (N <= 0 || K <= 0) return hipSuccess;
    const CacheDev none = {};
    float *h = const_cast<float *>(h_out);              // not written without a cache
    if (m.dtype == RNNLM_BF16)
        launch_query_typed<bf16_t, false>(m, rows, B_dev, N, K, splits, query_word, row_of_query, h, lse_rows,
                                          base_score, logprob, none, nullptr, stream);
    else
        launch_query_typed<float, false>(m, rows, B_dev, N, K, splits, query_word, row_of_query, h, lse_rows,
                                         base_score, logprob, none, nullptr, stream);
    return hipGetLastError();
}

hipError_t launch_query_cached(const ModelDev &m, const CacheDev &c, int rows, const int32_t *n_unique, int N, int K,
                               SplitInfo splits, const int32_t *query_word, const int32_t *inverse,
                               const int32_t *rep, float *h_out, const float *base_score, float *score,
                               hipStream_t stream) {
    if (N <= 0 || K <= 0) return hipSuccess;
    if (m.dtype == RNNLM_BF16)
        launch_query_typed<bf16_t, true>(m, rows, n_unique, N, K, splits, query_word, inverse, h_out, nullptr,
                                         base_score, score, c, rep, stream);
    else
        launch_query_typed<float, true>(m, rows, n_unique, N, K, splits, query_word, inverse, h_out, nullptr,
                                        base_score, score, c, rep, stream);
    return hipGetLastError();
}

}  // namespace rnnlm
