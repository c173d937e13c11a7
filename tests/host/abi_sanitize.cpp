// Host code of the library under AddressSanitizer and UndefinedBehaviorSanitizer: the argument checks
// of every entry point that rejects its arguments before any device call, and the Huffman builder
// (host code throughout).  Built host-only, no device is touched.  Prints "ok".
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rnnlm.h"
#include "rnnlm_diag.h"

#define CHECK(cond)                                                      \
    do {                                                                 \
        if (!(cond)) {                                                   \
            std::printf("FAILED line %d: %s\n", __LINE__, #cond);        \
            return 1;                                                    \
        }                                                                \
    } while (0)

static uint64_t state = 0x9e3779b97f4a7c15ull;
static uint32_t next_u32() {
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}

// Kraft sum of the code lengths must be exactly 1, the offsets must partition the entries, every
// entry must name an inner node, every path must start at the root.
static int check_tree(int V, const std::vector<int32_t> &off, const std::vector<int32_t> &entry) {
    long double kraft = 0;
    for (int v = 0; v < V; ++v) {
        const int len = off[v + 1] - off[v];
        CHECK(len >= 1 && len <= V - 1);
        kraft += 1.0L / (long double)(1ull << (len < 63 ? len : 63));
        CHECK((entry[off[v]] & 0x7fffffff) == V - 2);
        for (int i = off[v]; i < off[v + 1]; ++i) CHECK((entry[i] & 0x7fffffff) <= V - 2);
    }
    if (V <= 60) CHECK(kraft > 1.0L - 1e-12L && kraft < 1.0L + 1e-12L);
    return 0;
}

static int huffman_cases() {
    const int sizes[] = {2, 3, 4, 5, 7, 64, 1000, 4099};
    for (int V : sizes)
        for (int kind = 0; kind < 4; ++kind) {
            std::vector<double> f(V);
            for (int v = 0; v < V; ++v)
                f[v] = kind == 0 ? 1.0 : kind == 1 ? 1.0 / (v + 1.0) : kind == 2 ? (double)(next_u32() % 4) : (double)(1ull << (v % 40));
            std::vector<int32_t> off(V + 1);
            size_t needed = 0;
            CHECK(rnnlm_huffman_build(V, f.data(), off.data(), nullptr, 0, &needed) == RNNLM_ERANGE);
            CHECK(needed >= (size_t)V && off[V] == (int32_t)needed);
            std::vector<int32_t> entry(needed);
            if (needed > 1) {                     // one entry short: refused, nothing written past the end
                std::vector<int32_t> tight(needed - 1);
                CHECK(rnnlm_huffman_build(V, f.data(), off.data(), tight.data(), needed - 1, nullptr) == RNNLM_ERANGE);
            }
            CHECK(rnnlm_huffman_build(V, f.data(), off.data(), entry.data(), needed, &needed) == RNNLM_OK);
            if (check_tree(V, off, entry)) return 1;
        }
    double one = 1.0, bad[2] = {1.0, -1.0};
    int32_t off2[3];
    CHECK(rnnlm_huffman_build(1, &one, off2, nullptr, 0, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_huffman_build(2, nullptr, off2, nullptr, 0, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_huffman_build(2, bad, nullptr, nullptr, 0, nullptr) == RNNLM_EINVAL);
    return 0;
}

static int argument_checks() {
    rnnlm_model *out = nullptr;
    float buf[64] = {0};
    int32_t ibuf[64] = {0};
    uint64_t ids[8] = {0};
    void *p = buf;
    CHECK(rnnlm_load(0, 8, RNNLM_F32, p, p, p, buf, 4, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_load(8, 0, RNNLM_F32, p, p, p, buf, 4, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_load(8, 8, 7, p, p, p, buf, 4, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_load(8, 8, RNNLM_F32, nullptr, p, p, buf, 4, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_load(8, 8, RNNLM_F32, p, p, p, buf, 0, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_load(8, 8, RNNLM_F32, p, p, p, buf, 4, nullptr) == RNNLM_EINVAL);
    CHECK(out == nullptr);
    CHECK(rnnlm_free(nullptr) == RNNLM_OK);
    CHECK(rnnlm_model_share(nullptr, 4, &out) == RNNLM_EINVAL);
    CHECK(rnnlm_set_option(nullptr, 1, 0) == RNNLM_EINVAL);
    CHECK(rnnlm_step(nullptr, 1, 1, ibuf, buf, ibuf, nullptr, 0, buf, buf, nullptr) == RNNLM_EINVAL);
    size_t need = rnnlm_dedup_workspace_bytes(4);
    CHECK(need > 0);
    CHECK(rnnlm_dedup(ids, -1, ibuf, ibuf, ibuf, p, 1 << 20, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_dedup(nullptr, 4, ibuf, ibuf, ibuf, p, 1 << 20, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_dedup(ids, 4, ibuf, ibuf, ibuf, p, 8, nullptr) == RNNLM_EWORKSPACE);
    CHECK(rnnlm_dedup(ids, (1 << 28) + 1, ibuf, ibuf, ibuf, p, 1 << 20, nullptr) == RNNLM_ERANGE);
    CHECK(rnnlm_dedup_static(ids, -1, ibuf, ibuf, ibuf, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_dedup_static(nullptr, 4, ibuf, ibuf, ibuf, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_dedup_static(ids, RNNLM_DEDUP_STATIC_MAX_N + 1, ibuf, ibuf, ibuf, nullptr) == RNNLM_ERANGE);
    float ms = 0.f, us = 0.f;
    CHECK(rnnlm_time_outproj(nullptr, 1, nullptr, 1, nullptr, &ms) == RNNLM_EINVAL);
    CHECK(rnnlm_time_empty_launch(0, nullptr, &us) == RNNLM_EINVAL);
    CHECK(rnnlm_time_empty_launch(10, nullptr, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_outproj_kernel_name(nullptr, 4) == nullptr);
    double tf = 0;
    CHECK(rnnlm_probe_mfma_rate(2, 0, 1, &tf, nullptr) == RNNLM_EINVAL);
    CHECK(rnnlm_probe_mfma_rate(0, 0, 1001, &tf, nullptr) == RNNLM_EINVAL);
    return 0;
}

int main() {
    if (huffman_cases()) return 1;
    if (argument_checks()) return 1;
    std::printf("ok\n");
    return 0;
}
