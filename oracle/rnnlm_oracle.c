/*
 * CPU oracle for the batched RNNLM step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, scalar fp64 evaluation of what one step computes, written from the
 * definitions and sharing nothing with the GPU library.  Only the tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it; the product path never does.
 *
 * What is computed (one "history" = previous word + previous hidden vector; the paper's
 * RNNLM context, Section 4.1):
 *
 *   grouping   RnnlmProb's lookup (Table 1, steps 1-3 and 14): a key that was seen before
 *              reuses the stored result; a new key gets the next index, in order of first
 *              appearance (Table 1 step 10 numbers new entries sequentially).
 *   hidden     h'[j] = 1 / (1 + exp(-(U[w_prev][j] + sum_i W[j][i] h[i])))    -- the
 *              one-hidden-layer recurrent LM that Section 2 builds on (the paper prints
 *              no equations; this is the standard form, logistic activation, no hidden
 *              bias).
 *   output     z[v] = bias[v] + sum_j O[j][v] h'[j];  the probability of word v is
 *              normalised over all V words (the cost Section 2.1 names):
 *              logp[v] = z[v] - (m + log sum_u exp(z[u] - m)),  m = max_u z[u].
 *   query      only logp at the queried words is returned.
 *   cache      the same lookup kept between steps (Table 1 as a whole; Sections 4.2, 5.3),
 *              the score difference handed back after it, and the packed 8-byte index of
 *              Section 3.2: oracle_step_cached, oracle_pack_ids further down.
 *   tree       the hierarchical output layer of Section 2.1 (Huffman tree over the words,
 *              probability = product of sigmoids along the path): oracle_huffman_build,
 *              oracle_hs_step further down.
 *   index      IndexTable and its inverse (Section 3.2, Table 1 steps 5, 7-12): contexts stored
 *              by value, found again by content: oracle_index_* further down.
 *
 * Everything is summed left to right in double.  Weights arrive as float (bf16 models
 * pass values that are exact in float) and are widened exactly.  h' is never rounded
 * before the output layer uses it.  Rows are independent; OpenMP may spread rows over
 * threads, which changes no result.
 *
 * Pinned by tests/test_oracle_pins.py (closed forms, brute force, library routines).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Grouping of equal keys.  rep[u] = first raw index holding the u-th distinct key,
 * inverse[n] = group of raw query n.  Returns the number of distinct keys. */
int oracle_dedup(const uint64_t *keys, int N, int32_t *rep, int32_t *inverse)
{
    int U = 0;
    for (int n = 0; n < N; ++n) {
        int found = -1;
        for (int u = 0; u < U; ++u) {          /* "if Cache[I] exists" */
            if (keys[rep[u]] == keys[n]) { found = u; break; }
        }
        if (found < 0) {                       /* new entry takes the next index */
            rep[U] = n;
            found = U;
            ++U;
        }
        inverse[n] = found;
    }
    return U;
}

/* Hidden update of one row.  W is [H][H] row-major, W[j][i] multiplies h[i]. */
static void hidden_row(int H, const float *Urow, const float *W, const float *h_in, double *h_out)
{
    for (int j = 0; j < H; ++j) {
        double a = (double)Urow[j];
        for (int i = 0; i < H; ++i)
            a += (double)W[(size_t)j * H + i] * (double)h_in[i];
        h_out[j] = 1.0 / (1.0 + exp(-a));
    }
}

/* All V logits of one row.  O is [H][V] row-major.  The j-loop is outermost so memory is
 * walked in order; each z[v] still receives its H terms in the order j = 0..H-1. */
static void logits_row(int V, int H, const float *O, const float *bias, const double *h, double *z)
{
    for (int v = 0; v < V; ++v)
        z[v] = bias ? (double)bias[v] : 0.0;
    for (int j = 0; j < H; ++j) {
        const float *Oj = O + (size_t)j * V;
        double hj = h[j];
        for (int v = 0; v < V; ++v)
            z[v] += (double)Oj[v] * hj;
    }
}

static double log_sum_exp(int V, const double *z)
{
    double m = z[0];
    for (int v = 1; v < V; ++v)
        if (z[v] > m) m = z[v];
    double s = 0.0;
    for (int v = 0; v < V; ++v)
        s += exp(z[v] - m);
    return m + log(s);
}

/*
 * One step for B rows and N raw queries.
 *   prev[B], h_in[B][H] (float), query[N][K]; row_of_query[N] maps a raw query to its row
 *   (NULL: N == B and query n belongs to row n).
 * Outputs (double): h_out[B][H], lse[B] (may be NULL), logprob[N][K].
 * full_logp (may be NULL): [B][V] log-probabilities of every word, for the sum-to-one pin.
 * Returns 0, or -1 on a word id outside [0,V) / a row index outside [0,B).
 */
int oracle_step(int V, int H, int B, int K, int N,
                const float *U, const float *W, const float *O, const float *bias,
                const int32_t *prev, const float *h_in,
                const int32_t *query, const int32_t *row_of_query,
                double *h_out, double *lse, double *logprob, double *full_logp,
                int num_threads)
{
    for (int b = 0; b < B; ++b)
        if (prev[b] < 0 || prev[b] >= V) return -1;
    for (int n = 0; n < N; ++n) {
        int r = row_of_query ? row_of_query[n] : n;
        if (r < 0 || r >= B) return -1;
        for (int k = 0; k < K; ++k)
            if (query[(size_t)n * K + k] < 0 || query[(size_t)n * K + k] >= V) return -1;
    }
    (void)num_threads;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
    int bad = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *z = (double *)malloc((size_t)V * sizeof(double));
        if (!z) {
#pragma omp atomic write
            bad = 1;
            continue;
        }
        double *h = h_out + (size_t)b * H;
        hidden_row(H, U + (size_t)prev[b] * H, W, h_in + (size_t)b * H, h);
        logits_row(V, H, O, bias, h, z);
        double l = log_sum_exp(V, z);
        if (lse) lse[b] = l;
        if (full_logp)
            for (int v = 0; v < V; ++v) full_logp[(size_t)b * V + v] = z[v] - l;
        /* answer every raw query that points at this row */
        for (int n = 0; n < N; ++n) {
            int r = row_of_query ? row_of_query[n] : n;
            if (r != b) continue;
            for (int k = 0; k < K; ++k)
                logprob[(size_t)n * K + k] = z[query[(size_t)n * K + k]] - l;
        }
        free(z);
    }
    return bad ? -2 : 0;
}

/* ------------------------------------------------------------------------------------
 * RnnlmProb with a cache that outlives one step (Table 1; Section 4.2), keyed by the 8-byte
 * history index of Section 3.2.  The cache holds at most `capacity` entries (the size
 * boundary of Section 5.3); the paper removes nothing from a bounded cache, so once it is
 * full a new history is still computed and answered but not kept.  An entry stores what the
 * output of a history depends on: its updated hidden vector h' and the normaliser lse.
 */
typedef struct oracle_cache {
    int H, capacity, count;
    uint64_t *keys;     /* [capacity] */
    double *h;          /* [capacity][H] */
    double *lse;        /* [capacity] */
    long long lookups, hits, misses, unstored;   /* running totals over distinct histories */
} oracle_cache;

oracle_cache *oracle_cache_new(int H, int capacity)
{
    if (H <= 0 || capacity < 0) return NULL;
    oracle_cache *c = (oracle_cache *)calloc(1, sizeof(oracle_cache));
    if (!c) return NULL;
    c->H = H;
    c->capacity = capacity;
    size_t cap = capacity > 0 ? (size_t)capacity : 1;
    c->keys = (uint64_t *)malloc(cap * sizeof(uint64_t));
    c->h = (double *)malloc(cap * (size_t)H * sizeof(double));
    c->lse = (double *)malloc(cap * sizeof(double));
    if (!c->keys || !c->h || !c->lse) { free(c->keys); free(c->h); free(c->lse); free(c); return NULL; }
    return c;
}

void oracle_cache_free(oracle_cache *c)
{
    if (!c) return;
    free(c->keys); free(c->h); free(c->lse); free(c);
}

/* Start of an utterance: forget everything (Section 4.2 resets per utterance). */
void oracle_cache_reset(oracle_cache *c)
{
    c->count = 0;
    c->lookups = c->hits = c->misses = c->unstored = 0;
}

void oracle_cache_stats(const oracle_cache *c, long long out[5])
{
    out[0] = c->count; out[1] = c->lookups; out[2] = c->hits; out[3] = c->misses; out[4] = c->unstored;
}

/*
 * One step over N raw queries with the cache (c == NULL: no cache outlives the step).
 *   ids[N], prev[N], h_in[N][H], query[N][K]; base_score[N][K] or NULL.
 * Walks the queries in order, as RnnlmProb is called: a history met earlier in this step
 * reuses that result (steps 2-3); a history found in the cache takes the stored (h', lse)
 * whatever prev/h_in say now; any other history is computed from the prev/h_in of its first
 * query and, while there is room, stored (step 14).  The arithmetic of the computed
 * histories is independent of the walk, so it is evaluated for all of them together.
 * Outputs: rep[U], inverse[N] as oracle_dedup; h_out[U][H], lse[U] in group order;
 *   score[n][k] = logp(query[n][k] | history n) - base_score[n][k]
 * (Section 4.2, last paragraph: the value handed back is the difference to the short-span
 * n-gram score); step_stats = {distinct, found in cache, computed, entries afterwards}.
 * Returns the number of distinct histories, or < 0 as oracle_step.
 */
int oracle_step_cached(oracle_cache *c, int V, int H, int N, int K,
                       const float *U, const float *W, const float *O, const float *bias,
                       const uint64_t *ids, const int32_t *prev, const float *h_in,
                       const int32_t *query, const float *base_score,
                       int32_t *rep, int32_t *inverse,
                       double *h_out, double *lse, double *score, int32_t step_stats[4],
                       int num_threads)
{
    if (c && c->H != H) return -1;
    int nu = 0, nhit = 0, nmiss = 0;
    int32_t *entry = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));  /* cache entry or -1 */
    int32_t *miss_rows = (int32_t *)malloc((size_t)(N > 0 ? N : 1) * sizeof(int32_t));
    if (!entry || !miss_rows) { free(entry); free(miss_rows); return -2; }
    for (int n = 0; n < N; ++n) {
        int u = -1;
        for (int t = 0; t < nu; ++t)
            if (ids[rep[t]] == ids[n]) { u = t; break; }
        if (u < 0) {
            u = nu++;
            rep[u] = n;
            entry[u] = -1;
            if (c)
                for (int e = 0; e < c->count; ++e)
                    if (c->keys[e] == ids[n]) { entry[u] = e; break; }
            if (entry[u] >= 0) ++nhit;
            else miss_rows[nmiss++] = u;
        }
        inverse[n] = u;
    }
    /* ComputeRnnlm for the histories that were not cached */
    int rc = 0;
    if (nmiss > 0) {
        int32_t *mprev = (int32_t *)malloc((size_t)nmiss * sizeof(int32_t));
        float *mh = (float *)malloc((size_t)nmiss * H * sizeof(float));
        double *mho = (double *)malloc((size_t)nmiss * H * sizeof(double));
        double *mlse = (double *)malloc((size_t)nmiss * sizeof(double));
        if (!mprev || !mh || !mho || !mlse) rc = -2;
        if (rc == 0) {
            for (int m = 0; m < nmiss; ++m) {
                int n = rep[miss_rows[m]];
                mprev[m] = prev[n];
                for (int i = 0; i < H; ++i) mh[(size_t)m * H + i] = h_in[(size_t)n * H + i];
            }
            rc = oracle_step(V, H, nmiss, 0, 0, U, W, O, bias, mprev, mh, NULL, NULL, mho, mlse, NULL, NULL,
                             num_threads);
        }
        if (rc == 0)
            for (int m = 0; m < nmiss; ++m) {
                int u = miss_rows[m];
                for (int j = 0; j < H; ++j) h_out[(size_t)u * H + j] = mho[(size_t)m * H + j];
                lse[u] = mlse[m];
            }
        free(mprev); free(mh); free(mho); free(mlse);
    }
    if (rc != 0) { free(entry); free(miss_rows); return rc; }
    /* cached histories: the stored values; new ones: stored in order of first appearance */
    for (int u = 0; u < nu; ++u) {
        if (entry[u] >= 0) {
            for (int j = 0; j < H; ++j) h_out[(size_t)u * H + j] = c->h[(size_t)entry[u] * H + j];
            lse[u] = c->lse[entry[u]];
        } else if (c) {
            if (c->count < c->capacity) {
                int e = c->count++;
                c->keys[e] = ids[rep[u]];
                for (int j = 0; j < H; ++j) c->h[(size_t)e * H + j] = h_out[(size_t)u * H + j];
                c->lse[e] = lse[u];
            } else {
                ++c->unstored;
            }
        }
    }
    if (c) { c->lookups += nu; c->hits += nhit; c->misses += nmiss; }
    /* the queried words */
    for (int n = 0; n < N && rc == 0; ++n) {
        const double *h = h_out + (size_t)inverse[n] * H;
        for (int k = 0; k < K; ++k) {
            int q = query[(size_t)n * K + k];
            if (q < 0 || q >= V) { rc = -1; break; }
            double z = bias ? (double)bias[q] : 0.0;
            for (int j = 0; j < H; ++j) z += (double)O[(size_t)j * V + q] * h[j];
            double p = z - lse[inverse[n]];
            if (base_score) p -= (double)base_score[(size_t)n * K + k];
            score[(size_t)n * K + k] = p;
        }
    }
    if (step_stats) {
        step_stats[0] = nu; step_stats[1] = nhit; step_stats[2] = nmiss; step_stats[3] = c ? c->count : 0;
    }
    free(entry); free(miss_rows);
    return rc != 0 ? rc : nu;
}

/* The 8-byte value of Section 3.2: the RNNLM context index and the index of the small
 * (graph-building) LM in one number, context index in the high half. */
void oracle_pack_ids(const uint32_t *ctx, const uint32_t *small_lm, int N, uint64_t *ids)
{
    for (int n = 0; n < N; ++n) ids[n] = ((uint64_t)ctx[n] << 32) | (uint64_t)small_lm[n];
}

/* ------------------------------------------------------------------------------------
 * IndexTable and its inverse (Section 3.2; Table 1 steps 5 and 7-12): a context -- the word it
 * ends in and its hidden vector (Section 4.1) -- is stored once and stands for its index from
 * then on.  Two contexts are the same when the word and every bit of the hidden vector agree.
 * Indices are handed out in the order of first storage (step 10).  The table holds at most
 * `capacity` contexts; one that does not fit gets the index 0xFFFFFFFF and is not stored.
 */
#include <string.h>

typedef struct oracle_index {
    int H, capacity, count;
    int32_t *word;      /* [capacity] */
    float *h;           /* [capacity][H] */
    long long lookups, found, unstored;    /* running totals over the distinct contexts of each call */
} oracle_index;

oracle_index *oracle_index_new(int H, int capacity)
{
    if (H <= 0 || capacity < 0) return NULL;
    oracle_index *t = (oracle_index *)calloc(1, sizeof(oracle_index));
    if (!t) return NULL;
    t->H = H;
    t->capacity = capacity;
    size_t cap = capacity > 0 ? (size_t)capacity : 1;
    t->word = (int32_t *)malloc(cap * sizeof(int32_t));
    t->h = (float *)malloc(cap * (size_t)H * sizeof(float));
    if (!t->word || !t->h) { free(t->word); free(t->h); free(t); return NULL; }
    return t;
}

void oracle_index_free(oracle_index *t)
{
    if (!t) return;
    free(t->word); free(t->h); free(t);
}

void oracle_index_reset(oracle_index *t)
{
    t->count = 0;
    t->lookups = t->found = t->unstored = 0;
}

void oracle_index_stats(const oracle_index *t, long long out[4])
{
    out[0] = t->count; out[1] = t->lookups; out[2] = t->found; out[3] = t->unstored;
}

static int same_context(int H, int32_t w1, const float *h1, int32_t w2, const float *h2)
{
    return w1 == w2 && memcmp(h1, h2, (size_t)H * sizeof(float)) == 0;
}

/* IndexTable^-1 for N contexts given by value, in order: the index of a context already in the
 * table, else the next free index (and the context is stored).  A context that occurs several
 * times in one call counts once in the totals. */
void oracle_index_intern(oracle_index *t, int N, const int32_t *word, const float *h, uint32_t *index)
{
    int H = t->H;
    for (int n = 0; n < N; ++n) {
        const float *hn = h + (size_t)n * H;
        int seen_in_call = 0;
        for (int p = 0; p < n && !seen_in_call; ++p)
            if (same_context(H, word[n], hn, word[p], h + (size_t)p * H)) { index[n] = index[p]; seen_in_call = 1; }
        if (seen_in_call) continue;
        ++t->lookups;
        int e = -1;
        for (int i = 0; i < t->count; ++i)
            if (same_context(H, word[n], hn, t->word[i], t->h + (size_t)i * H)) { e = i; break; }
        if (e >= 0) {
            ++t->found;
        } else if (t->count < t->capacity) {
            e = t->count++;
            t->word[e] = word[n];
            memcpy(t->h + (size_t)e * H, hn, (size_t)H * sizeof(float));
        } else {
            ++t->unstored;
        }
        index[n] = e >= 0 ? (uint32_t)e : 0xFFFFFFFFu;
    }
}

/* IndexTable[c]: the stored context of every index.  Returns -1 on an index that is not held. */
int oracle_index_fetch(const oracle_index *t, int N, const uint32_t *index, int32_t *word, float *h)
{
    for (int n = 0; n < N; ++n) {
        if (index[n] >= (uint32_t)t->count) return -1;
        word[n] = t->word[index[n]];
        memcpy(h + (size_t)n * t->H, t->h + (size_t)index[n] * t->H, (size_t)t->H * sizeof(float));
    }
    return 0;
}

/* ------------------------------------------------------------------------------------
 * Hierarchical softmax (Section 2.1): the output layer is a binary tree with the words at the
 * leaves, built by Huffman's method from the word frequencies (frequent words get short
 * codes); the probability of a word is normalised only over the nodes on the path from the
 * root to the word.  The paper prints no formula; this is the standard form: every inner node
 * i has a vector theta_i, and
 *     p(w | h') = prod over the path nodes i of sigmoid(+-theta_i . h'),
 * + for a step to the child with code bit 0, - for code bit 1, so that the two children of a
 * node share its probability mass and the leaves sum to one.
 *
 * Huffman's method by its definition: keep the set of live subtrees; while more than one is left,
 * take out the two of least weight and put back a new inner node that has them as children and
 * the sum of their weights as weight.  The set is a binary heap ordered by (weight, node number),
 * where words are nodes 0 .. V-1 and the n-th inner node created is node V + n: among equal
 * weights the lower number is taken first, i.e. a word before an inner node, words in order of
 * their id, inner nodes in order of creation.  (Any tie rule gives an optimal code; this one is
 * fixed so that exactly one tree is right.)  The first of the two taken becomes the child with
 * code bit 0.  Codes are then read off by walking down from the root (node 2V-2).
 * Output per word: its path from the root down as entries inner-node index (0 .. V-2, the root
 * is V-2) | code bit << 31.
 * Returns the number of entries, or -1 (V < 2, a negative frequency, out of memory), or
 * -(needed) - 1 when `capacity` is too small.
 */
typedef struct { double w; int32_t node; } hs_item;

static int hs_before(hs_item a, hs_item b)
{
    return a.w < b.w || (a.w == b.w && a.node < b.node);
}

static void hs_push(hs_item *heap, int *n, hs_item x)
{
    int i = (*n)++;
    while (i > 0 && hs_before(x, heap[(i - 1) / 2])) {
        heap[i] = heap[(i - 1) / 2];
        i = (i - 1) / 2;
    }
    heap[i] = x;
}

static hs_item hs_pop(hs_item *heap, int *n)
{
    hs_item top = heap[0], last = heap[--(*n)];
    int i = 0;
    for (;;) {
        int c = 2 * i + 1;
        if (c >= *n) break;
        if (c + 1 < *n && hs_before(heap[c + 1], heap[c])) ++c;
        if (!hs_before(heap[c], last)) break;
        heap[i] = heap[c];
        i = c;
    }
    if (*n > 0) heap[i] = last;
    return top;
}

/* A node waiting to be visited on the walk down: how deep it is and the entry (parent's inner
 * index | code bit << 31) that leads to it. */
typedef struct { int32_t node, depth; uint32_t via; } hs_visit;

long long oracle_huffman_build(int V, const double *freq, int32_t *path_off, int32_t *path_entry,
                               long long capacity)
{
    if (V < 2) return -1;
    for (int v = 0; v < V; ++v)
        if (!(freq[v] >= 0.0)) return -1;
    hs_item *heap = (hs_item *)malloc((size_t)V * sizeof(hs_item));
    int32_t *child = (int32_t *)malloc((size_t)(V - 1) * 2 * sizeof(int32_t));   /* child[2n + bit] of inner node n */
    hs_visit *todo = (hs_visit *)malloc((size_t)(V + 1) * sizeof(hs_visit));
    uint32_t *trail = (uint32_t *)malloc((size_t)V * sizeof(uint32_t));          /* entries from the root to here */
    if (!heap || !child || !todo || !trail) {
        free(heap); free(child); free(todo); free(trail);
        return -1;
    }
    int live = 0;
    for (int v = 0; v < V; ++v) {
        hs_item x = { freq[v], v };
        hs_push(heap, &live, x);
    }
    for (int n = 0; live > 1; ++n) {
        hs_item a = hs_pop(heap, &live), b = hs_pop(heap, &live);
        child[2 * n + 0] = a.node;
        child[2 * n + 1] = b.node;
        hs_item merged = { a.w + b.w, V + n };
        hs_push(heap, &live, merged);
    }
    /* Two walks down from the root, depth first: the first measures the code lengths (a word's
     * offset needs the lengths of all words with smaller ids), the second writes the entries. */
    long long total = 0;
    for (int pass = 0; pass < 2; ++pass) {
        int top = 0;
        todo[top].node = 2 * V - 2; todo[top].depth = 0; todo[top].via = 0; ++top;
        while (top > 0) {
            const hs_visit at = todo[--top];
            if (at.depth > 0) trail[at.depth - 1] = at.via;
            if (at.node < V) {                                 /* a word: trail[0 .. depth) is its path */
                if (pass == 0) path_off[at.node + 1] = at.depth;
                else if (total <= capacity)
                    for (int e = 0; e < at.depth; ++e) path_entry[path_off[at.node] + e] = (int32_t)trail[e];
                continue;
            }
            const int n = at.node - V;
            for (int bit = 1; bit >= 0; --bit) {               /* bit 0 is visited first */
                todo[top].node = child[2 * n + bit];
                todo[top].depth = at.depth + 1;
                todo[top].via = (uint32_t)n | ((uint32_t)bit << 31);
                ++top;
            }
        }
        if (pass == 0) {
            path_off[0] = 0;
            for (int v = 0; v < V; ++v) path_off[v + 1] += path_off[v];
            total = path_off[V];
        }
    }
    free(heap); free(child); free(todo); free(trail);
    return total <= capacity ? total : -total - 1;
}

static double log_sigmoid(double z)
{
    return z >= 0.0 ? -log1p(exp(-z)) : z - log1p(exp(z));
}

/* log p(word | h) along its path; theta is [V-1][H]. */
static double hs_logp(int H, const float *theta, const int32_t *path_off, const int32_t *path_entry,
                      int word, const double *h)
{
    double lp = 0.0;
    for (int e = path_off[word]; e < path_off[word + 1]; ++e) {
        uint32_t entry = (uint32_t)path_entry[e];
        const float *th = theta + (size_t)(entry & 0x7FFFFFFFu) * H;
        double x = 0.0;
        for (int j = 0; j < H; ++j) x += (double)th[j] * h[j];
        lp += log_sigmoid((entry >> 31) ? -x : x);
    }
    return lp;
}

/*
 * One step with the hierarchical output layer: arguments as oracle_step, with theta and the
 * paths in place of O and bias.  full_logp (may be NULL): [B][V] log-probabilities of every
 * word, for the sum-to-one pin.
 */
int oracle_hs_step(int V, int H, int B, int K, int N,
                   const float *U, const float *W, const float *theta,
                   const int32_t *path_off, const int32_t *path_entry,
                   const int32_t *prev, const float *h_in,
                   const int32_t *query, const int32_t *row_of_query,
                   double *h_out, double *logprob, double *full_logp, int num_threads)
{
    for (int b = 0; b < B; ++b)
        if (prev[b] < 0 || prev[b] >= V) return -1;
    for (int n = 0; n < N; ++n) {
        int r = row_of_query ? row_of_query[n] : n;
        if (r < 0 || r >= B) return -1;
        for (int k = 0; k < K; ++k)
            if (query[(size_t)n * K + k] < 0 || query[(size_t)n * K + k] >= V) return -1;
    }
    (void)num_threads;
#ifdef _OPENMP
    if (num_threads > 0) omp_set_num_threads(num_threads);
#endif
#pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        double *h = h_out + (size_t)b * H;
        hidden_row(H, U + (size_t)prev[b] * H, W, h_in + (size_t)b * H, h);
        if (full_logp)
            for (int v = 0; v < V; ++v)
                full_logp[(size_t)b * V + v] = hs_logp(H, theta, path_off, path_entry, v, h);
    }
#pragma omp parallel for schedule(dynamic, 16)
    for (int n = 0; n < N; ++n) {
        int r = row_of_query ? row_of_query[n] : n;
        for (int k = 0; k < K; ++k)
            logprob[(size_t)n * K + k] =
                hs_logp(H, theta, path_off, path_entry, query[(size_t)n * K + k], h_out + (size_t)r * H);
    }
    return 0;
}

/*
 * Table 1 as the paper runs it: RnnlmProb with its cache (Sections 3.2, 4.2) around a ComputeRnnlm
 * whose output layer is the hierarchical one (Section 2.1).  The walk over the raw queries is that
 * of oracle_step_cached; what a history's answers are made of is its updated hidden vector alone
 * (a path needs no normaliser), so that is all the cache keeps.  c == NULL: nothing outlives the
 * step.  Outputs: rep[U], inverse[N]; h_out[U][H] in group order;
 *   score[n][k] = log p(query[n][k] | history n) - base_score[n][k];
 * step_stats = {distinct, found in cache, computed, entries afterwards}.
 * Returns the number of distinct histories, -1 on a word id outside [0, V), -2 without memory.
 */
int oracle_hs_step_cached(oracle_cache *c, int V, int H, int N, int K,
                          const float *U, const float *W, const float *theta,
                          const int32_t *path_off, const int32_t *path_entry,
                          const uint64_t *ids, const int32_t *prev, const float *h_in,
                          const int32_t *query, const float *base_score,
                          int32_t *rep, int32_t *inverse, double *h_out, double *score, int32_t step_stats[4])
{
    if (c && c->H != H) return -1;
    for (int n = 0; n < N; ++n) {
        if (prev[n] < 0 || prev[n] >= V) return -1;
        for (int k = 0; k < K; ++k)
            if (query[(size_t)n * K + k] < 0 || query[(size_t)n * K + k] >= V) return -1;
    }
    int nu = 0, nhit = 0, nmiss = 0;
    for (int n = 0; n < N; ++n) {
        int u = -1;
        for (int t = 0; t < nu; ++t)                      /* met earlier in this step? */
            if (ids[rep[t]] == ids[n]) { u = t; break; }
        if (u < 0) {
            u = nu++;
            rep[u] = n;
            int e = -1;
            if (c)
                for (int i = 0; i < c->count; ++i)
                    if (c->keys[i] == ids[n]) { e = i; break; }
            double *h = h_out + (size_t)u * H;
            if (e >= 0) {                                  /* "Cache[I] exists": the stored context, whatever prev / h_in say now */
                ++nhit;
                for (int j = 0; j < H; ++j) h[j] = c->h[(size_t)e * H + j];
            } else {                                       /* ComputeRnnlm, then store while there is room */
                ++nmiss;
                hidden_row(H, U + (size_t)prev[n] * H, W, h_in + (size_t)n * H, h);
                if (c) {
                    if (c->count < c->capacity) {
                        int slot = c->count++;
                        c->keys[slot] = ids[n];
                        for (int j = 0; j < H; ++j) c->h[(size_t)slot * H + j] = h[j];
                        c->lse[slot] = 0.0;
                    } else {
                        ++c->unstored;
                    }
                }
            }
        }
        inverse[n] = u;
    }
    if (c) { c->lookups += nu; c->hits += nhit; c->misses += nmiss; }
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            double p = hs_logp(H, theta, path_off, path_entry, query[(size_t)n * K + k], h_out + (size_t)inverse[n] * H);
            if (base_score) p -= (double)base_score[(size_t)n * K + k];
            score[(size_t)n * K + k] = p;
        }
    if (step_stats) {
        step_stats[0] = nu; step_stats[1] = nhit; step_stats[2] = nmiss; step_stats[3] = c ? c->count : 0;
    }
    return nu;
}

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
