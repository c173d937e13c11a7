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
        if (!z) { bad = 1; continue; }
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

int oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
