/* The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: every entry point on small
 * seeded inputs, with the sizes that stress its indexing (one row, one word, ragged row maps, a
 * cache and an index table that fill up, trees with ties).  Values are checked elsewhere; here the
 * sanitizers watch the memory accesses and the arithmetic.  Prints "ok". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle_cache oracle_cache;
typedef struct oracle_index oracle_index;
int oracle_dedup(const uint64_t *keys, int N, int32_t *rep, int32_t *inverse);
int oracle_step(int V, int H, int B, int K, int N, const float *U, const float *W, const float *O,
                const float *bias, const int32_t *prev, const float *h_in, const int32_t *query,
                const int32_t *row_of_query, double *h_out, double *lse, double *logprob,
                double *full_logp, int num_threads);
oracle_cache *oracle_cache_new(int H, int capacity);
void oracle_cache_free(oracle_cache *c);
void oracle_cache_reset(oracle_cache *c);
void oracle_cache_stats(const oracle_cache *c, long long out[5]);
int oracle_step_cached(oracle_cache *c, int V, int H, int N, int K, const float *U, const float *W,
                       const float *O, const float *bias, const uint64_t *ids, const int32_t *prev,
                       const float *h_in, const int32_t *query, const float *base_score, int32_t *rep,
                       int32_t *inverse, double *h_out, double *lse, double *score,
                       int32_t step_stats[4], int num_threads);
void oracle_pack_ids(const uint32_t *ctx, const uint32_t *small_lm, int N, uint64_t *ids);
oracle_index *oracle_index_new(int H, int capacity);
void oracle_index_free(oracle_index *t);
void oracle_index_reset(oracle_index *t);
void oracle_index_stats(const oracle_index *t, long long out[4]);
void oracle_index_intern(oracle_index *t, int N, const int32_t *word, const float *h, uint32_t *index);
int oracle_index_fetch(const oracle_index *t, int N, const uint32_t *index, int32_t *word, float *h);
long long oracle_huffman_build(int V, const double *freq, int32_t *path_off, int32_t *path_entry,
                               long long capacity);
int oracle_hs_step(int V, int H, int B, int K, int N, const float *U, const float *W, const float *theta,
                   const int32_t *path_off, const int32_t *path_entry, const int32_t *prev,
                   const float *h_in, const int32_t *query, const int32_t *row_of_query, double *h_out,
                   double *logprob, double *full_logp, int num_threads);
int oracle_hs_step_cached(oracle_cache *c, int V, int H, int N, int K, const float *U, const float *W,
                          const float *theta, const int32_t *path_off, const int32_t *path_entry,
                          const uint64_t *ids, const int32_t *prev, const float *h_in, const int32_t *query,
                          const float *base_score, int32_t *rep, int32_t *inverse, double *h_out, double *score,
                          int32_t step_stats[4]);
int oracle_max_threads(void);

#define CHECK(cond)                                               \
    do {                                                          \
        if (!(cond)) {                                            \
            printf("FAILED line %d: %s\n", __LINE__, #cond);      \
            exit(1);                                              \
        }                                                         \
    } while (0)

static uint64_t state = 0x243f6a8885a308d3ull;
static uint32_t next_u32(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(state >> 33);
}
static float next_float(float scale) { return scale * ((float)(next_u32() % 20001) / 10000.0f - 1.0f); }
static float *floats(size_t n, float scale)
{
    float *a = (float *)malloc((n ? n : 1) * sizeof(float));   /* exact size: an overrun is seen */
    for (size_t i = 0; i < n; ++i) a[i] = next_float(scale);
    return a;
}
static int32_t *ints(size_t n, int below)
{
    int32_t *a = (int32_t *)malloc((n ? n : 1) * sizeof(int32_t));
    for (size_t i = 0; i < n; ++i) a[i] = (int32_t)(next_u32() % (uint32_t)below);
    return a;
}
static double *doubles(size_t n) { return (double *)malloc((n ? n : 1) * sizeof(double)); }

static void full_softmax_case(int V, int H, int B, int K, int N, int with_map, int with_bias, int with_full)
{
    float *U = floats((size_t)V * H, 0.3f), *W = floats((size_t)H * H, 0.3f), *O = floats((size_t)H * V, 0.3f);
    float *bias = with_bias ? floats((size_t)V, 1.0f) : NULL, *h_in = floats((size_t)B * H, 1.0f);
    int32_t *prev = ints((size_t)B, V), *query = ints((size_t)N * K, V), *map = with_map ? ints((size_t)N, B) : NULL;
    double *h_out = doubles((size_t)B * H), *lse = doubles((size_t)B), *lp = doubles((size_t)N * K);
    double *full = with_full ? doubles((size_t)B * V) : NULL;
    CHECK(oracle_step(V, H, B, K, with_map ? N : B, U, W, O, bias, prev, h_in, query, map, h_out, lse, lp, full, 2) == 0);
    for (int i = 0; i < (with_map ? N : B) * K; ++i) CHECK(lp[i] <= 0.0 && isfinite(lp[i]));
    if (N * K > 0) {                                   /* a word id out of range is refused, nothing is read */
        query[0] = V;
        CHECK(oracle_step(V, H, B, K, with_map ? N : B, U, W, O, bias, prev, h_in, query, map, h_out, lse, lp, full, 1) == -1);
    }
    free(U); free(W); free(O); free(bias); free(h_in); free(prev); free(query); free(map);
    free(h_out); free(lse); free(lp); free(full);
}

static void cached_case(int V, int H, int N, int K, int capacity, int distinct)
{
    float *U = floats((size_t)V * H, 0.3f), *W = floats((size_t)H * H, 0.3f), *O = floats((size_t)H * V, 0.3f);
    oracle_cache *c = capacity >= 0 ? oracle_cache_new(H, capacity) : NULL;
    for (int step = 0; step < 4; ++step) {
        float *h_in = floats((size_t)N * H, 1.0f), *base = (step & 1) ? floats((size_t)N * K, 2.0f) : NULL;
        int32_t *prev = ints((size_t)N, V), *query = ints((size_t)N * K, V);
        uint64_t *ids = (uint64_t *)malloc((size_t)(N ? N : 1) * sizeof(uint64_t));
        for (int n = 0; n < N; ++n) ids[n] = 1000u * (uint64_t)(step / 2) + next_u32() % (uint32_t)distinct;
        int32_t *rep = (int32_t *)malloc((size_t)(N ? N : 1) * sizeof(int32_t)), *inv = (int32_t *)malloc((size_t)(N ? N : 1) * sizeof(int32_t));
        double *h_out = doubles((size_t)N * H), *lse = doubles((size_t)N), *score = doubles((size_t)N * K);
        int32_t stats[4];
        int nu = oracle_step_cached(c, V, H, N, K, U, W, O, NULL, ids, prev, h_in, query, base, rep, inv, h_out, lse, score, stats, 2);
        CHECK(nu >= (N > 0) && nu <= N && stats[0] == nu);
        int32_t *rep2 = (int32_t *)malloc((size_t)(N ? N : 1) * sizeof(int32_t)), *inv2 = (int32_t *)malloc((size_t)(N ? N : 1) * sizeof(int32_t));
        CHECK(oracle_dedup(ids, N, rep2, inv2) == nu);
        CHECK(memcmp(rep, rep2, (size_t)nu * sizeof(int32_t)) == 0 && memcmp(inv, inv2, (size_t)N * sizeof(int32_t)) == 0);
        free(h_in); free(base); free(prev); free(query); free(ids); free(rep); free(inv); free(rep2); free(inv2);
        free(h_out); free(lse); free(score);
    }
    if (c) {
        long long st[5];
        oracle_cache_stats(c, st);
        CHECK(st[0] <= capacity);
        oracle_cache_reset(c);
        oracle_cache_stats(c, st);
        CHECK(st[0] == 0);
    }
    oracle_cache_free(c);
    free(U); free(W); free(O);
}

static void index_case(int H, int capacity, int N)
{
    oracle_index *t = oracle_index_new(H, capacity);
    CHECK(t != NULL);
    for (int round = 0; round < 3; ++round) {
        float *h = floats((size_t)N * H, 1.0f);
        int32_t *word = ints((size_t)N, 5);
        for (int n = 1; n < N; n += 3) {                 /* repeats inside the call */
            memcpy(h + (size_t)n * H, h + (size_t)(n - 1) * H, (size_t)H * sizeof(float));
            word[n] = word[n - 1];
        }
        uint32_t *index = (uint32_t *)malloc((size_t)(N ? N : 1) * sizeof(uint32_t));
        oracle_index_intern(t, N, word, h, index);
        int stored = 0;
        uint32_t *kept = (uint32_t *)malloc((size_t)(N ? N : 1) * sizeof(uint32_t));
        for (int n = 0; n < N; ++n)
            if (index[n] != 0xffffffffu) kept[stored++] = index[n];
        int32_t *w2 = (int32_t *)malloc((size_t)(stored ? stored : 1) * sizeof(int32_t));
        float *h2 = (float *)malloc((size_t)(stored ? stored : 1) * H * sizeof(float));
        CHECK(oracle_index_fetch(t, stored, kept, w2, h2) == 0);
        uint32_t beyond = 0x7fffffffu;
        CHECK(oracle_index_fetch(t, 1, &beyond, w2, h2) == -1 || stored == 0);
        free(h); free(word); free(index); free(kept); free(w2); free(h2);
    }
    long long st[4];
    oracle_index_stats(t, st);
    CHECK(st[0] <= capacity);
    oracle_index_reset(t);
    oracle_index_free(t);
}

static void tree_case(int V, int H, int B, int K, int kind)
{
    double *freq = doubles((size_t)V);
    for (int v = 0; v < V; ++v)
        freq[v] = kind == 0 ? 1.0 : kind == 1 ? 1.0 / (v + 1.0) : kind == 2 ? (double)(next_u32() % 3) : ldexp(1.0, v % 50);
    int32_t *off = (int32_t *)malloc((size_t)(V + 1) * sizeof(int32_t));
    long long need = -oracle_huffman_build(V, freq, off, NULL, 0) - 1;   /* too small: the size, negated */
    CHECK(need >= V && off[V] == need);
    if (need > 1) {                                       /* one entry short: nothing is written */
        int32_t *tight = (int32_t *)malloc((size_t)(need - 1) * sizeof(int32_t));
        CHECK(oracle_huffman_build(V, freq, off, tight, need - 1) == -need - 1);
        free(tight);
    }
    int32_t *entry = (int32_t *)malloc((size_t)need * sizeof(int32_t));
    CHECK(oracle_huffman_build(V, freq, off, entry, need) == need);
    float *U = floats((size_t)V * H, 0.3f), *W = floats((size_t)H * H, 0.3f), *theta = floats((size_t)(V - 1) * H, 0.5f);
    float *h_in = floats((size_t)B * H, 1.0f);
    int32_t *prev = ints((size_t)B, V), *query = ints((size_t)B * K, V);
    double *h_out = doubles((size_t)B * H), *lp = doubles((size_t)B * K), *full = doubles((size_t)B * V);
    CHECK(oracle_hs_step(V, H, B, K, B, U, W, theta, off, entry, prev, h_in, query, NULL, h_out, lp, full, 2) == 0);
    for (int b = 0; b < B; ++b) {                         /* a tree gives a distribution: the sanitizers' run checks it too */
        double total = 0;
        for (int v = 0; v < V; ++v) total += exp(full[(size_t)b * V + v]);
        CHECK(fabs(total - 1.0) < 1e-9);
    }
    /* the same rows as raw queries through a cache that fills up (ids repeat: b / 2) */
    {
        oracle_cache *c = oracle_cache_new(H, 1);
        uint64_t *ids = (uint64_t *)malloc((size_t)B * sizeof(uint64_t));
        for (int b = 0; b < B; ++b) ids[b] = 77u + (uint64_t)(b / 2);
        int32_t *rep = (int32_t *)malloc((size_t)B * sizeof(int32_t)), *inv = (int32_t *)malloc((size_t)B * sizeof(int32_t));
        double *h2 = doubles((size_t)B * H), *score = doubles((size_t)B * K);
        int32_t stats[4];
        for (int pass = 0; pass < 2; ++pass) {
            int nu = oracle_hs_step_cached(pass ? c : NULL, V, H, B, K, U, W, theta, off, entry, ids, prev, h_in, query, NULL,
                                           rep, inv, h2, score, stats);
            CHECK(nu == (B + 1) / 2 && stats[0] == nu && stats[3] == (pass ? 1 : 0));
        }
        oracle_cache_free(c);
        free(ids); free(rep); free(inv); free(h2); free(score);
    }
    freq[0] = -1.0;
    CHECK(oracle_huffman_build(V, freq, off, entry, need) == -1);
    free(freq); free(off); free(entry); free(U); free(W); free(theta); free(h_in); free(prev); free(query);
    free(h_out); free(lp); free(full);
}

int main(void)
{
    CHECK(oracle_max_threads() >= 1);
    full_softmax_case(1, 1, 1, 1, 1, 0, 0, 1);
    full_softmax_case(7, 3, 5, 2, 5, 0, 1, 1);
    full_softmax_case(33, 8, 4, 3, 11, 1, 1, 0);
    full_softmax_case(129, 17, 9, 0, 9, 0, 0, 0);
    full_softmax_case(50, 5, 0, 2, 0, 0, 0, 0);
    cached_case(40, 6, 12, 3, 5, 9);        /* the cache fills up */
    cached_case(40, 6, 12, 3, 0, 9);        /* a cache that keeps nothing */
    cached_case(40, 6, 12, 3, -1, 4);       /* no cache */
    cached_case(40, 6, 1, 1, 100, 1);
    cached_case(40, 6, 0, 2, 100, 1);
    uint32_t ctx[3] = {0u, 0xffffffffu, 7u}, lm[3] = {0xffffffffu, 0u, 9u};
    uint64_t ids[3];
    oracle_pack_ids(ctx, lm, 3, ids);
    CHECK(ids[0] == 0xffffffffull && ids[1] == 0xffffffff00000000ull && ids[2] == ((7ull << 32) | 9ull));
    index_case(4, 6, 5);                    /* fills up in the second call */
    index_case(3, 0, 4);
    index_case(5, 100, 0);
    const int sizes[] = {2, 3, 4, 5, 9, 64, 257};
    for (unsigned i = 0; i < sizeof sizes / sizeof sizes[0]; ++i)
        for (int kind = 0; kind < 4; ++kind) tree_case(sizes[i], 4, 3, 2, kind);
    printf("ok\n");
    return 0;
}
