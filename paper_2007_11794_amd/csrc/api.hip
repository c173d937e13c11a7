// C ABI of librnnlm: argument checks, model set-up, and the order of kernel launches.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <new>
#include <vector>

#include "rnnlm_internal.h"

using namespace rnnlm;

namespace {

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

#define HIP_TRY(expr)                                  \
    do {                                               \
        hipError_t e_ = (expr);                        \
        if (e_ != hipSuccess) {                        \
            status = (e_ == hipErrorOutOfMemory) ? RNNLM_ENOMEM : RNNLM_EDEVICE; \
            goto fail;                                 \
        }                                              \
    } while (0)

size_t elem_size(int dtype) { return dtype == RNNLM_BF16 ? 2 : 4; }

bool use_fixed_offset(const rnnlm_model *m) {
    if (m->lse_mode == 1) return false;
    if (m->lse_mode == 2) return true;
    return m->fixed_ok != 0;
}

// The model as the hidden update sees it: a copy of the hidden block that the following kernel does not
// read is not written (null pointer).  Full softmax: the row-ordered copy when the output projection
// takes the fragment-ordered one (launch sized for `rows` rows); hierarchical layer: neither (the path
// kernel reads h_out itself).
ModelDev recur_view(const rnnlm_model *m, int rows) {
    ModelDev v = m->dev;
    if (v.dtype != RNNLM_BF16) return v;
    if (v.hs) { v.d = nullptr; v.dfrag = nullptr; return v; }
    if (!outproj_reads_row_order(v, rows, use_fixed_offset(m), m->outproj_kernel)) v.d = nullptr;
    return v;
}

// What belongs to one handle alone: its scratch blocks, its flag, its events.
void free_scratch(rnnlm_model *m) {
    ModelDev &d = m->dev;
    (void)hipFree(d.d);
    (void)hipFree(d.dfrag);
    (void)hipFree(d.part);
    (void)hipFree(d.flag);
    (void)hipFree(d.d3);
    d.d = d.dfrag = d.d3 = nullptr; d.part = nullptr; d.flag = nullptr;
    if (m->ev0) (void)hipEventDestroy(m->ev0);
    if (m->ev1) (void)hipEventDestroy(m->ev1);
    m->ev0 = m->ev1 = nullptr;
}

// The weights and what rnnlm_load derived from them: shared by every handle on the model.
void free_weights(rnnlm_model *m) {
    ModelDev &d = m->dev;
    (void)hipFree(const_cast<void *>(d.U));
    (void)hipFree(const_cast<void *>(d.W));
    (void)hipFree(const_cast<void *>(d.Ot));
    (void)hipFree(const_cast<float *>(d.half_rowsum_W));
    (void)hipFree(const_cast<float *>(d.bias));
    (void)hipFree(const_cast<float *>(d.half_colsum_O));
    (void)hipFree(const_cast<float *>(d.cvec2));
    (void)hipFree(const_cast<float *>(d.cvec2_fixed));
    (void)hipFree(const_cast<void *>(d.Ot3));
    (void)hipFree(const_cast<void *>(d.Ofrag));
    (void)hipFree(const_cast<void *>(d.Theta));
    (void)hipFree(const_cast<int32_t *>(d.path_off));
    (void)hipFree(const_cast<int32_t *>(d.path_entry));
}

void free_dev(rnnlm_model *m) {
    free_scratch(m);
    free_weights(m);
}

std::mutex g_handles_mutex;        // guards rnnlm_model::owner / handles / released of every model

// Scratch of one handle for batches of up to max_Bp rows (a multiple of 256): hidden block in row and
// fragment order, log-sum-exp partials, three-term block (fp32 full-softmax models), flag, events.
// On failure the caller releases with free_scratch.
int alloc_scratch(rnnlm_model *m, int max_Bp, bool with_partials, bool with_split3) {
    int status = RNNLM_OK;
    ModelDev &d = m->dev;
    const size_t es = elem_size(d.dtype), block = (size_t)max_Bp * d.Hp * es;
    void *p;
    HIP_TRY(hipMalloc(&p, block)); d.d = p;
    HIP_TRY(hipMemset(d.d, 0, block));
    HIP_TRY(hipMalloc(&p, 4)); d.flag = static_cast<int *>(p);
    HIP_TRY(hipMemset(d.flag, 0, 4));
    if (d.dtype == RNNLM_BF16) {
        HIP_TRY(hipMalloc(&p, block)); d.dfrag = p;
        HIP_TRY(hipMemset(d.dfrag, 0, block));
    }
    if (with_partials) {
        HIP_TRY(hipMalloc(&p, (size_t)max_Bp * kMaxSplits * sizeof(float2))); d.part = static_cast<float2 *>(p);
        HIP_TRY(hipMemset(d.part, 0, (size_t)max_Bp * kMaxSplits * sizeof(float2)));
    }
    if (with_split3) {
        HIP_TRY(hipMalloc(&p, (size_t)max_Bp * 3 * d.Hp * 2)); d.d3 = p;
        HIP_TRY(hipMemset(d.d3, 0, (size_t)max_Bp * 3 * d.Hp * 2));
    }
    HIP_TRY(hipEventCreate(&m->ev0));
    HIP_TRY(hipEventCreate(&m->ev1));
    return RNNLM_OK;
fail:
    return status;
}

// Do [a, a + n) and [b, b + n) floats share an element?
bool ranges_overlap(const float *a, const float *b, size_t n) {
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b), bytes = n * sizeof(float);
    return x < y + bytes && y < x + bytes;
}

double widen_host(const void *p, size_t i, int dtype) {
    if (dtype == RNNLM_BF16) {
        uint32_t u = (uint32_t)static_cast<const uint16_t *>(p)[i] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    return (double)static_cast<const float *>(p)[i];
}

// Device copies of what the hidden update needs (U, W zero-padded to Hp, half row sums of W) and
// the handle's scratch.  On failure the caller releases with free_dev.
int upload_recurrent(rnnlm_model *m, int V, int H, int Hp, int dtype, const void *U, const void *W, int max_Bp,
                     bool with_partials, bool with_split3) {
    int status = RNNLM_OK;
    const size_t es = elem_size(dtype);
    ModelDev &d = m->dev;
    std::vector<float> hrs;
    void *p;
    HIP_TRY(hipMalloc(&p, (size_t)V * Hp * es)); d.U = p;
    HIP_TRY(hipMalloc(&p, (size_t)Hp * Hp * es)); d.W = p;
    HIP_TRY(hipMalloc(&p, (size_t)Hp * 4)); d.half_rowsum_W = static_cast<float *>(p);
    status = alloc_scratch(m, max_Bp, with_partials, with_split3);
    if (status != RNNLM_OK) return status;
    HIP_TRY(hipMemset(const_cast<void *>(d.U), 0, (size_t)V * Hp * es));
    HIP_TRY(hipMemset(const_cast<void *>(d.W), 0, (size_t)Hp * Hp * es));
    HIP_TRY(hipMemcpy2D(const_cast<void *>(d.U), Hp * es, U, H * es, H * es, V, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy2D(const_cast<void *>(d.W), Hp * es, W, H * es, H * es, H, hipMemcpyHostToDevice));
    // half row sums of W in fp64 on the host (H*H elements)
    hrs.assign(Hp, 0.f);
    for (int j = 0; j < H; ++j) {
        double sum = 0.0;
        for (int i = 0; i < H; ++i) sum += widen_host(W, (size_t)j * H + i, dtype);
        hrs[j] = (float)(0.5 * sum);
    }
    HIP_TRY(hipMemcpy(const_cast<float *>(d.half_rowsum_W), hrs.data(), (size_t)Hp * 4, hipMemcpyHostToDevice));
    return RNNLM_OK;
fail:
    return status;
}

// Device memory of a CacheDev (hash table, stores, counters, per-call scratch for up to nb
// histories); shared by the step's cache and the index table.  Null pointers are left for
// release_cache_dev on failure.
int alloc_cache_dev(CacheDev &d, int capacity, int H, size_t nb, bool with_lse) {
    int status = RNNLM_OK;
    d.capacity = capacity;
    d.table_size = 64;
    while (d.table_size < 2 * capacity) d.table_size <<= 1;
    d.H = H;
    const size_t cap1 = capacity > 0 ? (size_t)capacity : 1;
    void *p;
    HIP_TRY(hipMalloc(&p, (size_t)d.table_size * sizeof(CacheCell))); d.table = static_cast<CacheCell *>(p);
    HIP_TRY(hipMalloc(&p, cap1 * H * 4)); d.store_h = static_cast<float *>(p);
    HIP_TRY(hipMalloc(&p, 4)); d.n_entries = static_cast<int *>(p);
    HIP_TRY(hipMalloc(&p, 4 * sizeof(long long))); d.totals = static_cast<long long *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.entry_of = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.miss_of = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.miss_src = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.miss_dst = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, 4)); d.n_miss = static_cast<int *>(p);
    HIP_TRY(hipMalloc(&p, (nb / 1024 + 2) * 4)); d.block_total = static_cast<int *>(p);
    if (with_lse) {
        HIP_TRY(hipMalloc(&p, cap1 * 4)); d.store_lse = static_cast<float *>(p);
        HIP_TRY(hipMalloc(&p, nb * 4)); d.lse_rows = static_cast<float *>(p);
    }
    HIP_TRY(hipMemset(d.n_miss, 0, 4));
    return RNNLM_OK;
fail:
    return status;
}

void release_cache_dev(CacheDev &d) {
    (void)hipFree(d.table); (void)hipFree(d.store_h); (void)hipFree(d.store_lse); (void)hipFree(d.n_entries);
    (void)hipFree(d.totals); (void)hipFree(d.entry_of); (void)hipFree(d.miss_of); (void)hipFree(d.miss_src);
    (void)hipFree(d.miss_dst); (void)hipFree(d.lse_rows); (void)hipFree(d.n_miss); (void)hipFree(d.block_total);
}

int check_step_args(const rnnlm_model *model, int B, int K, int N, int hs = 0) {
    if (!model) return RNNLM_EINVAL;
    if (model->dev.hs != hs) return RNNLM_EINVAL;       // full-softmax and hierarchical models have their own steps
    if (B < 0 || K < 0 || N < 0) return RNNLM_EINVAL;
    if (B > model->max_B || N > model->max_B) return RNNLM_ERANGE;
    return RNNLM_OK;
}

}  // namespace

extern "C" {

const char *rnnlm_strerror(int status) {
    switch (status) {
        case RNNLM_OK: return "ok";
        case RNNLM_EINVAL: return "invalid argument";
        case RNNLM_ENOMEM: return "out of memory";
        case RNNLM_EDEVICE: return "HIP call failed";
        case RNNLM_ERANGE: return "batch larger than the model was loaded for, or size beyond the stated maximum";
        case RNNLM_EWORKSPACE: return "workspace too small or misaligned";
        default: return "unknown status";
    }
}

int rnnlm_load(int V, int H, int dtype, const void *U, const void *W, const void *O,
               const float *bias_or_null, int max_B, rnnlm_model **out) {
    if (!out) return RNNLM_EINVAL;
    *out = nullptr;
    if (!U || !W || !O) return RNNLM_EINVAL;
    if (V <= 0 || H <= 0 || max_B <= 0) return RNNLM_EINVAL;
    if (dtype != RNNLM_F32 && dtype != RNNLM_BF16) return RNNLM_EINVAL;
    if ((long long)V > (1ll << 30) || H > (1 << 16) || max_B > (1 << 24)) return RNNLM_EINVAL;

    rnnlm_model *m = new (std::nothrow) rnnlm_model();
    if (!m) return RNNLM_ENOMEM;
    memset(m, 0, sizeof(*m));
    int status = RNNLM_OK;
    const size_t es = elem_size(dtype);
    // bf16 models pad to at least 128 so that every Hp <= 512 fits the staged kernel
    const int Hp = (dtype == RNNLM_BF16 && H < 128) ? 128 : round_up(H, 64), Vp = round_up(V, 256);
    const int max_Bp = round_up(max_B, 256);
    ModelDev &d = m->dev;
    d.V = V; d.H = H; d.Hp = Hp; d.Vp = Vp; d.dtype = dtype;
    m->max_B = max_B; m->max_Bp = max_Bp;
    void *O_stage = nullptr;
    float *bias_stage = nullptr, *upper = nullptr, *lower = nullptr;
    std::vector<float> hu, hl;
    float max_upper = -INFINITY, min_lower = INFINITY;

    void *p;
    status = upload_recurrent(m, V, H, Hp, dtype, U, W, max_Bp, true, dtype == RNNLM_F32);
    if (status != RNNLM_OK) goto fail;
    HIP_TRY(hipMalloc(&p, (size_t)Vp * Hp * es)); d.Ot = p;
    HIP_TRY(hipMalloc(&p, (size_t)V * 4)); d.bias = static_cast<float *>(p);
    HIP_TRY(hipMalloc(&p, (size_t)V * 4)); d.half_colsum_O = static_cast<float *>(p);
    HIP_TRY(hipMalloc(&p, (size_t)Vp * 4)); d.cvec2 = static_cast<float *>(p);
    HIP_TRY(hipMalloc(&p, (size_t)Vp * 4)); d.cvec2_fixed = static_cast<float *>(p);

    // O: upload as given, transpose + pad on the device, column statistics
    HIP_TRY(hipMalloc(&O_stage, (size_t)H * V * es));
    HIP_TRY(hipMemcpy(O_stage, O, (size_t)H * V * es, hipMemcpyHostToDevice));
    if (bias_or_null) {
        HIP_TRY(hipMalloc(&p, (size_t)V * 4)); bias_stage = static_cast<float *>(p);
        HIP_TRY(hipMemcpy(bias_stage, bias_or_null, (size_t)V * 4, hipMemcpyHostToDevice));
    }
    HIP_TRY(hipMalloc(&p, (size_t)V * 4)); upper = static_cast<float *>(p);
    HIP_TRY(hipMalloc(&p, (size_t)V * 4)); lower = static_cast<float *>(p);
    HIP_TRY(launch_transpose_O(O_stage, const_cast<void *>(d.Ot), dtype, H, V, Hp, Vp, nullptr));
    HIP_TRY(launch_col_stats(O_stage, bias_stage, dtype, H, V, const_cast<float *>(d.half_colsum_O), upper,
                             lower, nullptr));
    hu.resize(V); hl.resize(V);
    HIP_TRY(hipMemcpy(hu.data(), upper, (size_t)V * 4, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(hl.data(), lower, (size_t)V * 4, hipMemcpyDeviceToHost));
    for (int v = 0; v < V; ++v) {
        if (!(hu[v] <= max_upper)) max_upper = hu[v];      // NaN-propagating max
        if (!(hl[v] >= min_lower)) min_lower = hl[v];
    }
    {
        // Every base-2 logit lies in [lo2, hi2] (margin covers fp32 rounding of the sums).
        const double hi2 = (double)max_upper * 1.4426950408889634, lo2 = (double)min_lower * 1.4426950408889634;
        const double margin = 0.01 + 1e-5 * (fabs(hi2) + fabs(lo2));
        d.m2_fixed = (float)(hi2 + margin);
        // usable when even the smallest possible term 2^(lo2 - m2) is a normal fp32 number
        m->fixed_ok = (isfinite(hi2) && isfinite(lo2) && (hi2 - lo2 + 2 * margin) < 100.0) ? 1 : 0;
        if (!isfinite(d.m2_fixed)) d.m2_fixed = 0.f;
    }
    HIP_TRY(launch_fill_cvec(bias_stage, d.half_colsum_O, V, Vp, d.m2_fixed, const_cast<float *>(d.bias),
                             const_cast<float *>(d.cvec2), const_cast<float *>(d.cvec2_fixed), nullptr));
    // operand-ordered copy for the weight-streaming kernels (few rows)
    HIP_TRY(hipMalloc(&p, (size_t)Vp * Hp * es)); d.Ofrag = p;
    HIP_TRY(launch_frag_weights(d.Ot, dtype, Vp, Hp, const_cast<void *>(d.Ofrag), nullptr));
    if (dtype == RNNLM_F32) {       // three-term bf16 split of the weights, scratch for that of the hidden block
        HIP_TRY(hipMalloc(&p, (size_t)Vp * 3 * Hp * 2)); d.Ot3 = p;
        HIP_TRY(launch_split3_weights(static_cast<const float *>(d.Ot), Vp, Hp, const_cast<void *>(d.Ot3), nullptr));
    }
    HIP_TRY(hipDeviceSynchronize());
    (void)hipFree(O_stage); (void)hipFree(bias_stage); (void)hipFree(upper); (void)hipFree(lower);
    (void)dedup_static_prepare();
    m->handles = 1;
    *out = m;
    return RNNLM_OK;

fail:
    (void)hipFree(O_stage); (void)hipFree(bias_stage); (void)hipFree(upper); (void)hipFree(lower);
    free_dev(m);
    delete m;
    (void)hipGetLastError();
    return status;
}

int rnnlm_free(rnnlm_model *model) {
    if (!model) return RNNLM_OK;
    hipError_t e = hipDeviceSynchronize();
    std::lock_guard<std::mutex> lock(g_handles_mutex);
    free_scratch(model);
    rnnlm_model *owner = model->owner ? model->owner : model;
    if (model == owner) owner->released = 1;
    --owner->handles;
    if (model != owner) delete model;
    if (owner->handles == 0) {             // the last handle on these weights is gone
        free_weights(owner);
        delete owner;
    }
    return e == hipSuccess ? RNNLM_OK : RNNLM_EDEVICE;
}

int rnnlm_model_share(const rnnlm_model *model, int max_B, rnnlm_model **out) {
    if (!out) return RNNLM_EINVAL;
    *out = nullptr;
    if (!model || max_B <= 0 || max_B > (1 << 24)) return RNNLM_EINVAL;
    rnnlm_model *m = new (std::nothrow) rnnlm_model();
    if (!m) return RNNLM_ENOMEM;
    *m = *model;                           // weights' pointers, shapes, options
    ModelDev &d = m->dev;
    d.d = d.dfrag = d.d3 = nullptr; d.part = nullptr; d.flag = nullptr;
    m->ev0 = m->ev1 = nullptr;
    m->max_B = max_B;
    m->max_Bp = round_up(max_B, 256);
    m->handles = 0; m->released = 0;
    int status = alloc_scratch(m, m->max_Bp, !d.hs, !d.hs && d.dtype == RNNLM_F32);
    if (status == RNNLM_OK && hipDeviceSynchronize() != hipSuccess) status = RNNLM_EDEVICE;
    if (status != RNNLM_OK) {
        free_scratch(m);
        delete m;
        (void)hipGetLastError();
        return status;
    }
    {
        std::lock_guard<std::mutex> lock(g_handles_mutex);
        rnnlm_model *owner = model->owner ? model->owner : const_cast<rnnlm_model *>(model);
        m->owner = owner;
        ++owner->handles;
    }
    *out = m;
    return RNNLM_OK;
}

int rnnlm_set_option(rnnlm_model *model, int option, int value) {
    if (!model) return RNNLM_EINVAL;
    switch (option) {
        case RNNLM_OPT_LSE_MODE:
            if (value < 0 || value > 2) return RNNLM_EINVAL;
            if (model->dev.hs || (value == 2 && !model->fixed_ok)) return RNNLM_EINVAL;
            model->lse_mode = value;
            return RNNLM_OK;
        case RNNLM_OPT_OUTPROJ_KERNEL:
            if (value < 0 || value > 6) return RNNLM_EINVAL;
            if (model->dev.hs) return RNNLM_EINVAL;
            if (value == 6 && !outproj_rowstream_supported(model->dev)) return RNNLM_EINVAL;
            if (value == 5 && outproj_stream_max_rows(model->dev) == 0) return RNNLM_EINVAL;
            if (value == 4 && !model->dev.Ot3) return RNNLM_EINVAL;
            if (value == 2 && !outproj_staged_supported(model->dev)) return RNNLM_EINVAL;
            model->outproj_kernel = value;
            return RNNLM_OK;
        default:
            return RNNLM_EINVAL;
    }
}

int rnnlm_last_error(rnnlm_model *model, void *hip_stream, int *flags) {
    if (!model || !flags) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int f = 0;
    if (hipMemcpyAsync(&f, model->dev.flag, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return RNNLM_EDEVICE;
    if (hipMemsetAsync(model->dev.flag, 0, 4, s) != hipSuccess) return RNNLM_EDEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return RNNLM_EDEVICE;
    *flags = f;
    return RNNLM_OK;
}

size_t rnnlm_dedup_workspace_bytes(int N) { return dedup_workspace_bytes(N); }

int rnnlm_dedup(const uint64_t *history_ids, int N, int32_t *rep, int32_t *inverse, int32_t *n_unique,
                void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (N < 0 || !n_unique) return RNNLM_EINVAL;
    if (N > 0 && (!history_ids || !rep || !inverse)) return RNNLM_EINVAL;
    if (N > (1 << 28)) return RNNLM_ERANGE;
    if (N > 0) {
        if (!workspace || workspace_bytes < dedup_workspace_bytes(N)) return RNNLM_EWORKSPACE;
        if (reinterpret_cast<uintptr_t>(workspace) & 15) return RNNLM_EWORKSPACE;
    }
    hipError_t e = launch_dedup(history_ids, N, rep, inverse, n_unique, workspace,
                                static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? RNNLM_OK : RNNLM_EDEVICE;
}

int rnnlm_step(const rnnlm_model *model, int B, int K, const int32_t *prev_word, const float *h_in,
               const int32_t *query_word, const int32_t *row_of_query_or_null, int N, float *h_out,
               float *logprob, void *hip_stream) {
    int rc = check_step_args(model, B, K, N);
    if (rc != RNNLM_OK) return rc;
    if (B > 0 && (!prev_word || !h_in || !h_out)) return RNNLM_EINVAL;
    if (N > 0 && K > 0 && (!query_word || !logprob)) return RNNLM_EINVAL;
    if (!row_of_query_or_null && N != B) return RNNLM_EINVAL;
    if (B > 0 && ranges_overlap(h_in, h_out, (size_t)B * model->dev.H)) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const ModelDev &d = model->dev;
    SplitInfo splits = fixed_split_info(1);
    if (launch_recur(recur_view(model, B), B, nullptr, nullptr, nullptr, prev_word, h_in, h_out, s) != hipSuccess) return RNNLM_EDEVICE;
    if (launch_outproj(d, B, nullptr, use_fixed_offset(model), model->outproj_kernel, &splits, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (launch_query(d, B, nullptr, N, K, splits, query_word, row_of_query_or_null, h_out, nullptr, nullptr, logprob, s) !=
        hipSuccess)
        return RNNLM_EDEVICE;
    return RNNLM_OK;
}

int rnnlm_step_dedup(const rnnlm_model *model, int N, int K, const uint64_t *history_ids,
                     const int32_t *prev_word, const float *h_in, const int32_t *query_word, int32_t *rep,
                     int32_t *inverse, int32_t *n_unique, float *h_out, float *logprob, void *workspace,
                     size_t workspace_bytes, void *hip_stream) {
    return rnnlm_step_cached(model, nullptr, N, K, history_ids, prev_word, h_in, query_word, nullptr, rep,
                             inverse, n_unique, h_out, logprob, nullptr, workspace, workspace_bytes, hip_stream);
}

int rnnlm_step_cached(const rnnlm_model *model, rnnlm_cache *cache, int N, int K, const uint64_t *history_ids,
                      const int32_t *prev_word, const float *h_in, const int32_t *query_word,
                      const float *base_score, int32_t *rep, int32_t *inverse, int32_t *n_unique, float *h_out,
                      float *score, int32_t *step_stats, void *workspace, size_t workspace_bytes,
                      void *hip_stream) {
    int rc = check_step_args(model, N, K, N, model ? model->dev.hs : 0);   // either kind of model
    if (rc != RNNLM_OK) return rc;
    if (!n_unique) return RNNLM_EINVAL;
    if (N > 0 && (!history_ids || !prev_word || !h_in || !rep || !inverse || !h_out)) return RNNLM_EINVAL;
    if (N > 0 && K > 0 && (!query_word || !score)) return RNNLM_EINVAL;
    if (N > 0 && ranges_overlap(h_in, h_out, (size_t)N * model->dev.H)) return RNNLM_EINVAL;
    if (cache && (cache->dev.H != model->dev.H || N > cache->max_B)) return RNNLM_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    // through a cache, few enough raw queries: grouping and lookup are one launch
    const bool one_launch = cache && N > 0 && N <= dedup_lookup_max_rows();
    if (one_launch) {
        if (!workspace || workspace_bytes < dedup_workspace_bytes(N)) return RNNLM_EWORKSPACE;   // as rnnlm_dedup
        if (reinterpret_cast<uintptr_t>(workspace) & 15) return RNNLM_EWORKSPACE;
        if (launch_dedup_lookup(cache->dev, history_ids, N, rep, inverse, n_unique, step_stats, s) != hipSuccess)
            return RNNLM_EDEVICE;
    } else {
        rc = rnnlm_dedup(history_ids, N, rep, inverse, n_unique, workspace, workspace_bytes, hip_stream);
        if (rc != RNNLM_OK) return rc;
    }
    const ModelDev &d = model->dev;
    SplitInfo splits = fixed_split_info(1);
    if (!cache) {
        if (N == 0) return RNNLM_OK;
        // Grids cover N rows; the kernels read the true number of rows from *n_unique.
        if (launch_recur(recur_view(model, N), N, n_unique, rep, nullptr, prev_word, h_in, h_out, s) != hipSuccess)
            return RNNLM_EDEVICE;
        if (d.hs) {                                         // hierarchical output layer: paths instead of the normaliser
            if (launch_hs_query(d, N, n_unique, N, K, query_word, inverse, h_out, base_score, score, s) != hipSuccess)
                return RNNLM_EDEVICE;
            return RNNLM_OK;
        }
        if (launch_outproj(d, N, n_unique, use_fixed_offset(model), model->outproj_kernel, &splits, s) !=
            hipSuccess)
            return RNNLM_EDEVICE;
        if (launch_query(d, N, n_unique, N, K, splits, query_word, inverse, h_out, nullptr, base_score, score,
                         s) != hipSuccess)
            return RNNLM_EDEVICE;
        return RNNLM_OK;
    }
    const CacheDev &c = cache->dev;
    if (!one_launch &&
        launch_cache_lookup(c, N, 4096, history_ids, rep, n_unique, step_stats, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (N == 0) return RNNLM_OK;
    // Only the histories the cache does not hold are computed: *c.n_miss rows, row r taken
    // from raw query c.miss_src[r], its hidden vector written to row c.miss_dst[r] of h_out.
    if (launch_recur(recur_view(model, N), N, c.n_miss, c.miss_src, c.miss_dst, prev_word, h_in, h_out, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (d.hs) {
        // Hierarchical output layer: what the cache keeps of a history is its hidden vector.  The
        // bookkeeping launch (stored vectors out to h_out, new ones in) leaves every distinct history's
        // vector in h_out; the path kernel then reads them there.
        if (launch_cache_commit(c, d, N, n_unique, splits, h_out, s) != hipSuccess) return RNNLM_EDEVICE;
        if (launch_hs_query(d, N, n_unique, N, K, query_word, inverse, h_out, base_score, score, s) != hipSuccess)
            return RNNLM_EDEVICE;
        return RNNLM_OK;
    }
    if (launch_outproj(d, N, c.n_miss, use_fixed_offset(model), model->outproj_kernel, &splits, s) != hipSuccess)
        return RNNLM_EDEVICE;
    // With words to score, the query kernel also does the cache's bookkeeping after the computation
    // (stored values out, new entries in): one launch less.
    if (K == 0) {
        if (launch_cache_commit(c, d, N, n_unique, splits, h_out, s) != hipSuccess) return RNNLM_EDEVICE;
        return RNNLM_OK;
    }
    if (launch_query_cached(d, c, N, n_unique, N, K, splits, query_word, inverse, rep, h_out, base_score, score,
                            s) != hipSuccess)
        return RNNLM_EDEVICE;
    return RNNLM_OK;
}

int rnnlm_cache_create(const rnnlm_model *model, int capacity, rnnlm_cache **out) {
    if (!out) return RNNLM_EINVAL;
    *out = nullptr;
    if (!model || capacity < 0) return RNNLM_EINVAL;
    if (capacity > (1 << 26)) return RNNLM_ERANGE;
    rnnlm_cache *c = new (std::nothrow) rnnlm_cache();
    if (!c) return RNNLM_ENOMEM;
    memset(c, 0, sizeof(*c));
    int status = RNNLM_OK;
    CacheDev &d = c->dev;
    c->max_B = model->max_B;
    status = alloc_cache_dev(d, capacity, model->dev.H, (size_t)model->max_B, true);
    if (status != RNNLM_OK) goto fail;
    HIP_TRY(launch_cache_reset(d, nullptr));
    HIP_TRY(hipDeviceSynchronize());
    *out = c;
    return RNNLM_OK;
fail:
    rnnlm_cache_free(c);
    (void)hipGetLastError();
    return status;
}

int rnnlm_cache_free(rnnlm_cache *cache) {
    if (!cache) return RNNLM_OK;
    hipError_t e = hipDeviceSynchronize();
    release_cache_dev(cache->dev);
    delete cache;
    return e == hipSuccess ? RNNLM_OK : RNNLM_EDEVICE;
}

int rnnlm_cache_reset(rnnlm_cache *cache, void *hip_stream) {
    if (!cache) return RNNLM_EINVAL;
    return launch_cache_reset(cache->dev, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? RNNLM_OK
                                                                                               : RNNLM_EDEVICE;
}

int rnnlm_cache_stats(rnnlm_cache *cache, void *hip_stream, int64_t out[5]) {
    if (!cache || !out) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int entries = 0;
    long long totals[4] = {0, 0, 0, 0};
    if (hipMemcpyAsync(&entries, cache->dev.n_entries, 4, hipMemcpyDeviceToHost, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (hipMemcpyAsync(totals, cache->dev.totals, sizeof(totals), hipMemcpyDeviceToHost, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return RNNLM_EDEVICE;
    out[0] = entries;
    for (int i = 0; i < 4; ++i) out[1 + i] = totals[i];
    return RNNLM_OK;
}

int rnnlm_hs_load(int V, int H, int dtype, const void *U, const void *W, const void *Theta,
                  const int32_t *path_offset, const int32_t *path_entry, int max_B, rnnlm_model **out) {
    if (!out) return RNNLM_EINVAL;
    *out = nullptr;
    if (!U || !W || !Theta || !path_offset || !path_entry) return RNNLM_EINVAL;
    if (V < 2 || H <= 0 || max_B <= 0) return RNNLM_EINVAL;
    if (dtype != RNNLM_F32 && dtype != RNNLM_BF16) return RNNLM_EINVAL;
    if ((long long)V > (1ll << 30) || H > (1 << 16) || max_B > (1 << 24)) return RNNLM_EINVAL;
    // the tree is walked on the device without further checks: every path must be non-empty
    // and name inner nodes only
    if (path_offset[0] != 0) return RNNLM_EINVAL;
    int longest = 0;
    for (int v = 0; v < V; ++v) {
        if (path_offset[v + 1] <= path_offset[v]) return RNNLM_EINVAL;
        if (path_offset[v + 1] - path_offset[v] > longest) longest = path_offset[v + 1] - path_offset[v];
    }
    const size_t entries = (size_t)path_offset[V];
    for (size_t e = 0; e < entries; ++e)
        if (((uint32_t)path_entry[e] & 0x7FFFFFFFu) >= (uint32_t)(V - 1)) return RNNLM_EINVAL;

    rnnlm_model *m = new (std::nothrow) rnnlm_model();
    if (!m) return RNNLM_ENOMEM;
    memset(m, 0, sizeof(*m));
    int status = RNNLM_OK;
    const size_t es = elem_size(dtype);
    const int Hp = (dtype == RNNLM_BF16 && H < 128) ? 128 : round_up(H, 64);
    const int max_Bp = round_up(max_B, 256);
    ModelDev &d = m->dev;
    d.V = V; d.H = H; d.Hp = Hp; d.Vp = round_up(V, 256); d.dtype = dtype; d.hs = 1; d.hs_max_len = longest;
    m->max_B = max_B; m->max_Bp = max_Bp;
    void *p;
    status = upload_recurrent(m, V, H, Hp, dtype, U, W, max_Bp, false, false);
    if (status != RNNLM_OK) goto fail;
    HIP_TRY(hipMalloc(&p, (size_t)(V - 1) * Hp * es)); d.Theta = p;
    HIP_TRY(hipMemset(p, 0, (size_t)(V - 1) * Hp * es));
    HIP_TRY(hipMemcpy2D(p, Hp * es, Theta, H * es, H * es, V - 1, hipMemcpyHostToDevice));
    HIP_TRY(hipMalloc(&p, ((size_t)V + 1) * 4)); d.path_off = static_cast<int32_t *>(p);
    HIP_TRY(hipMemcpy(p, path_offset, ((size_t)V + 1) * 4, hipMemcpyHostToDevice));
    HIP_TRY(hipMalloc(&p, entries * 4)); d.path_entry = static_cast<int32_t *>(p);
    HIP_TRY(hipMemcpy(p, path_entry, entries * 4, hipMemcpyHostToDevice));
    HIP_TRY(hipDeviceSynchronize());
    (void)dedup_static_prepare();
    m->handles = 1;
    *out = m;
    return RNNLM_OK;
fail:
    free_dev(m);
    delete m;
    (void)hipGetLastError();
    return status;
}

int rnnlm_hs_step(const rnnlm_model *model, int B, int K, const int32_t *prev_word, const float *h_in,
                  const int32_t *query_word, const int32_t *row_of_query_or_null, int N,
                  const float *base_score_or_null, float *h_out, float *logprob, void *hip_stream) {
    int rc = check_step_args(model, B, K, N, 1);
    if (rc != RNNLM_OK) return rc;
    if (B > 0 && (!prev_word || !h_in || !h_out)) return RNNLM_EINVAL;
    if (N > 0 && K > 0 && (!query_word || !logprob)) return RNNLM_EINVAL;
    if (!row_of_query_or_null && N != B) return RNNLM_EINVAL;
    if (B > 0 && ranges_overlap(h_in, h_out, (size_t)B * model->dev.H)) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const ModelDev &d = model->dev;
    if (launch_recur(recur_view(model, B), B, nullptr, nullptr, nullptr, prev_word, h_in, h_out, s) != hipSuccess) return RNNLM_EDEVICE;
    if (launch_hs_query(d, B, nullptr, N, K, query_word, row_of_query_or_null, h_out, base_score_or_null, logprob,
                        s) != hipSuccess)
        return RNNLM_EDEVICE;
    return RNNLM_OK;
}

int rnnlm_hs_time_query(const rnnlm_model *model, int B, int K, const int32_t *query_word,
                        const int32_t *row_of_query_or_null, int N, const float *h_out, float *logprob,
                        int repeats, void *hip_stream, float *ms_per_launch) {
    int rc = check_step_args(model, B, K, N, 1);
    if (rc != RNNLM_OK) return rc;
    if (!ms_per_launch || repeats <= 0 || B <= 0 || N <= 0 || K <= 0) return RNNLM_EINVAL;
    if (!query_word || !h_out || !logprob || (!row_of_query_or_null && N != B)) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (hipEventRecord(model->ev0, s) != hipSuccess) return RNNLM_EDEVICE;
    for (int i = 0; i < repeats; ++i)
        if (launch_hs_query(model->dev, B, nullptr, N, K, query_word, row_of_query_or_null, h_out, nullptr, logprob,
                            s) != hipSuccess)
            return RNNLM_EDEVICE;
    if (hipEventRecord(model->ev1, s) != hipSuccess) return RNNLM_EDEVICE;
    if (hipEventSynchronize(model->ev1) != hipSuccess) return RNNLM_EDEVICE;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, model->ev0, model->ev1) != hipSuccess) return RNNLM_EDEVICE;
    *ms_per_launch = ms / (float)repeats;
    return RNNLM_OK;
}

int rnnlm_index_create(int H, int capacity, int max_N, rnnlm_index_table **out) {
    if (!out) return RNNLM_EINVAL;
    *out = nullptr;
    if (H <= 0 || capacity < 0 || max_N <= 0) return RNNLM_EINVAL;
    if (capacity > (1 << 26) || max_N > (1 << 24) || H > (1 << 16)) return RNNLM_ERANGE;
    rnnlm_index_table *t = new (std::nothrow) rnnlm_index_table();
    if (!t) return RNNLM_ENOMEM;
    memset(t, 0, sizeof(*t));
    int status = RNNLM_OK;
    IndexDev &d = t->dev;
    t->max_N = max_N;
    const size_t nb = (size_t)max_N, cap1 = capacity > 0 ? (size_t)capacity : 1;
    void *p;
    status = alloc_cache_dev(d.c, capacity, H, nb, false);
    if (status != RNNLM_OK) goto fail;
    HIP_TRY(hipMalloc(&p, cap1 * 4)); d.store_word = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 8)); d.keys = static_cast<uint64_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.rep = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, nb * 4)); d.inverse = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, 4)); d.n_unique = static_cast<int32_t *>(p);
    HIP_TRY(hipMalloc(&p, dedup_workspace_bytes(max_N))); d.dedup_ws = p;
    HIP_TRY(hipMalloc(&p, 2 * sizeof(long long))); d.errors = static_cast<long long *>(p);
    HIP_TRY(launch_index_reset(d, nullptr));
    HIP_TRY(hipDeviceSynchronize());
    *out = t;
    return RNNLM_OK;
fail:
    rnnlm_index_free(t);
    (void)hipGetLastError();
    return status;
}

int rnnlm_index_free(rnnlm_index_table *table) {
    if (!table) return RNNLM_OK;
    hipError_t e = hipDeviceSynchronize();
    IndexDev &d = table->dev;
    release_cache_dev(d.c);
    (void)hipFree(d.store_word); (void)hipFree(d.keys); (void)hipFree(d.rep); (void)hipFree(d.inverse);
    (void)hipFree(d.n_unique); (void)hipFree(d.dedup_ws); (void)hipFree(d.errors);
    delete table;
    return e == hipSuccess ? RNNLM_OK : RNNLM_EDEVICE;
}

int rnnlm_index_reset(rnnlm_index_table *table, void *hip_stream) {
    if (!table) return RNNLM_EINVAL;
    return launch_index_reset(table->dev, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? RNNLM_OK
                                                                                               : RNNLM_EDEVICE;
}

int rnnlm_index_intern(rnnlm_index_table *table, int N, const int32_t *word, const float *h, uint32_t *index,
                       void *hip_stream) {
    if (!table || N < 0) return RNNLM_EINVAL;
    if (N > table->max_N) return RNNLM_ERANGE;
    if (N > 0 && (!word || !h || !index)) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    const IndexDev &d = table->dev;
    if (launch_context_hash(word, h, N, d.c.H, d.keys, s) != hipSuccess) return RNNLM_EDEVICE;
    if (launch_dedup(d.keys, N, d.rep, d.inverse, d.n_unique, d.dedup_ws, s) != hipSuccess) return RNNLM_EDEVICE;
    if (launch_cache_lookup(d.c, N, 1024, d.keys, d.rep, d.n_unique, nullptr, s) != hipSuccess) return RNNLM_EDEVICE;
    if (launch_index_commit(d, N, word, h, index, s) != hipSuccess) return RNNLM_EDEVICE;
    return RNNLM_OK;
}

int rnnlm_index_fetch(const rnnlm_index_table *table, int N, const uint32_t *index, int32_t *word, float *h,
                      void *hip_stream) {
    if (!table || N < 0) return RNNLM_EINVAL;
    if (N > 0 && (!index || !word || !h)) return RNNLM_EINVAL;
    return launch_index_fetch(table->dev, N, index, word, h, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? RNNLM_OK
               : RNNLM_EDEVICE;
}

int rnnlm_index_stats(rnnlm_index_table *table, void *hip_stream, int64_t out[6]) {
    if (!table || !out) return RNNLM_EINVAL;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    int entries = 0;
    long long totals[4] = {0, 0, 0, 0}, errors[2] = {0, 0};
    const IndexDev &d = table->dev;
    if (hipMemcpyAsync(&entries, d.c.n_entries, 4, hipMemcpyDeviceToHost, s) != hipSuccess) return RNNLM_EDEVICE;
    if (hipMemcpyAsync(totals, d.c.totals, sizeof(totals), hipMemcpyDeviceToHost, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (hipMemcpyAsync(errors, d.errors, sizeof(errors), hipMemcpyDeviceToHost, s) != hipSuccess)
        return RNNLM_EDEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return RNNLM_EDEVICE;
    out[0] = entries;
    out[1] = totals[0]; out[2] = totals[1]; out[3] = totals[3];
    out[4] = errors[0]; out[5] = errors[1];
    return RNNLM_OK;
}

int rnnlm_pack_ids(const uint32_t *ctx_idx, const uint32_t *small_lm_idx, int N, uint64_t *ids,
                   void *hip_stream) {
    if (N < 0) return RNNLM_EINVAL;
    if (N > 0 && (!ctx_idx || !small_lm_idx || !ids)) return RNNLM_EINVAL;
    return launch_pack_ids(ctx_idx, small_lm_idx, N, ids, static_cast<hipStream_t>(hip_stream)) == hipSuccess
               ? RNNLM_OK
               : RNNLM_EDEVICE;
}

const char *rnnlm_outproj_kernel_name(const rnnlm_model *model, int B) {
    if (!model || B <= 0 || B > model->max_B || model->dev.hs) return nullptr;
    return outproj_kernel_name(model->dev, B, use_fixed_offset(model), model->outproj_kernel);
}

int rnnlm_time_outproj(const rnnlm_model *model, int B, const int32_t *n_rows_dev, int repeats, void *hip_stream,
                       float *ms_per_launch) {
    if (!model || !ms_per_launch || repeats <= 0 || B <= 0 || model->dev.hs) return RNNLM_EINVAL;
    if (B > model->max_B) return RNNLM_ERANGE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    SplitInfo splits = fixed_split_info(1);
    const bool fixed = use_fixed_offset(model);
    if (hipEventRecord(model->ev0, s) != hipSuccess) return RNNLM_EDEVICE;
    for (int i = 0; i < repeats; ++i)
        if (launch_outproj(model->dev, B, n_rows_dev, fixed, model->outproj_kernel, &splits, s) != hipSuccess)
            return RNNLM_EDEVICE;
    if (hipEventRecord(model->ev1, s) != hipSuccess) return RNNLM_EDEVICE;
    if (hipEventSynchronize(model->ev1) != hipSuccess) return RNNLM_EDEVICE;
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, model->ev0, model->ev1) != hipSuccess) return RNNLM_EDEVICE;
    *ms_per_launch = ms / (float)repeats;
    return RNNLM_OK;
}

}  // extern "C"
