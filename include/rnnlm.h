/*
 * librnnlm -- batched RNNLM scoring step for network search, on one MI355X (gfx950).
 *
 * The search hands over, for every active hypothesis, a 64-bit history id, the previous
 * word, the previous hidden vector and the words it wants scored.  The library groups
 * identical histories, computes each distinct history once, and returns only the
 * log-probabilities that were asked for.  (The paper's RnnlmProb(w, c) -> (p, c') with a
 * cache of already computed contexts -- Section 4, Table 1 -- as one batched device step;
 * the full-vocabulary normalisation is the cost Section 2.1 describes.)
 *
 * Conventions
 *   - Plain C ABI.  Every function returns an rnnlm_status (0 = OK, < 0 = error) except
 *     where stated; nothing throws or aborts.
 *   - rnnlm_load takes HOST pointers and copies; the caller keeps its buffers.
 *   - rnnlm_dedup / rnnlm_step / rnnlm_step_dedup / rnnlm_step_cached / rnnlm_pack_ids /
 *     rnnlm_index_intern / rnnlm_index_fetch / rnnlm_hs_step take
 *     DEVICE pointers owned by the caller and are asynchronous on `hip_stream` (a
 *     hipStream_t passed as void*; NULL = the default stream).  No call here synchronises,
 *     allocates or frees device memory except rnnlm_load, rnnlm_hs_load, rnnlm_free, rnnlm_last_error,
 *     rnnlm_cache_create, rnnlm_cache_free, rnnlm_cache_stats, rnnlm_index_create,
 *     rnnlm_index_free and rnnlm_index_stats.
 *   - float / int32 / uint64 arrays are dense, row-major, naturally aligned; `h_in` and
 *     `h_out` rows must start on 16-byte boundaries when H is a multiple of 4 (any
 *     allocator's base alignment gives this).
 *   - A model handle may be used from one stream at a time (its scratch buffers are shared);
 *     rnnlm_model_share gives further handles on the same weights, each with scratch of its own,
 *     for further streams.
 *   - Host-checkable mistakes (NULL, negative sizes, B > max_B, short workspace) return
 *     before anything is launched.  Mistakes only visible on the device (a word id outside
 *     [0,V), a row index outside [0,B)) never cause an out-of-bounds access: the affected
 *     outputs become NaN and a sticky flag is raised, read by rnnlm_last_error.
 */
#ifndef RNNLM_H_
#define RNNLM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rnnlm_model rnnlm_model;       /* opaque, owned by the library */

enum rnnlm_dtype { RNNLM_F32 = 0, RNNLM_BF16 = 1 };

enum rnnlm_status {
    RNNLM_OK = 0,
    RNNLM_EINVAL = -1,        /* NULL pointer, bad size, unknown dtype or option */
    RNNLM_ENOMEM = -2,        /* device or host allocation failed */
    RNNLM_EDEVICE = -3,       /* a HIP call failed */
    RNNLM_ERANGE = -4,        /* B or N beyond what the model was loaded for, or beyond a stated maximum */
    RNNLM_EWORKSPACE = -5     /* workspace too small or misaligned */
};

/* Bits of the sticky device flag returned by rnnlm_last_error. */
enum rnnlm_device_flag {
    RNNLM_FLAG_BAD_PREV_WORD = 1,     /* prev_word outside [0,V): that row's outputs are NaN */
    RNNLM_FLAG_BAD_QUERY_WORD = 2,    /* query_word outside [0,V): that logprob is NaN */
    RNNLM_FLAG_BAD_ROW = 4            /* row_of_query outside [0,B): that query's logprobs are NaN */
};

/* Tunables for rnnlm_set_option. */
enum rnnlm_option {
    /* How the log-sum-exp over the vocabulary is taken (same mathematical result):
     * 0 = automatic (default): a fixed offset derived at load time from a bound on every
     *     logit when that bound is tight enough for fp32, else a running maximum;
     * 1 = always the running maximum;  2 = always the fixed offset (EINVAL if unusable). */
    RNNLM_OPT_LSE_MODE = 1,
    /* Which output-projection kernel: 0 = automatic (default), 1 = the plain any-shape
     * kernel, 2 = the LDS-staged kernel with the hidden block held in registers (bf16,
     * H <= 512), 3 = the LDS-tiled kernel for any hidden size and both types, 4 = (fp32 models)
     * the LDS-tiled kernel on the three-term bf16 split of both operands, fp32 accuracy at
     * bf16 matrix-core speed: the automatic choice for fp32 from 64 rows on, 5 = the weight-
     * streaming kernel for few rows, which reads a second, operand-ordered copy of the output
     * weights once per launch at memory speed (fp32 models: cut into three bf16 terms in registers,
     * fp32 accuracy): the automatic choice up to 64 rows when two launches suffice (the staged, the
     * eight-wave tiled and the three-term kernel also take it on the device, when a grouped or
     * cached step turns out to have that few rows and their LDS holds them).  One launch
     * serves as many rows as fit its LDS (bf16: 128 up to H = 576, 64 up to H = 1216, 32 up to
     * H = 2432; fp32: 128 up to H = 192, 64 up to H = 384, 32 up to H = 768); on request it takes
     * up to 128 rows in at most four launches, and larger batches go the automatic way,
     * 6 = (bf16 models) the kernel that sends only the weights through
     * LDS and takes the hidden rows straight into registers chunk by chunk: the automatic choice for
     * H > 512 from 256 rows on when batch and vocabulary give every compute unit a 256 x 256 tile (with
     * the running maximum it falls back to 3).
     * EINVAL if the model does not allow the choice. */
    RNNLM_OPT_OUTPROJ_KERNEL = 2
};

/* Human-readable text for a status code; never NULL; static storage. */
const char *rnnlm_strerror(int status);

/*
 * Load a model: V words, H hidden units (the recurrent LM of Section 2).
 *   dtype  RNNLM_F32: U, W, O are float.  RNNLM_BF16: they are uint16 bfloat16 bit
 *          patterns; products are accumulated in fp32 on the matrix cores.
 *   U      [V][H]  row w = input embedding of word w.
 *   W      [H][H]  W[j][i] multiplies h_in[i] in the pre-activation of unit j.
 *   O      [H][V]  output weights, z[v] = bias[v] + sum_j O[j][v] h'[j].
 *   bias   [V] float, or NULL for zero.
 *   max_B  largest number of rows (and of raw queries) any later call will pass.
 * All five are HOST pointers; the library uploads them and re-lays O out as [V][H].
 * *out receives the handle.  Synchronous.
 */
int rnnlm_load(int V, int H, int dtype, const void *U, const void *W, const void *O,
               const float *bias_or_null, int max_B, rnnlm_model **out);

/* Release a model handle and the device memory that belongs to it alone.  The weights go when the
 * last handle that shares them is released (any order).  NULL is a no-op.  Synchronises the device. */
int rnnlm_free(rnnlm_model *model);

/*
 * A further handle on the weights of `model` (either kind of model), with scratch buffers, sticky
 * flag and options of its own (options start as a copy): one loaded model can then serve several
 * streams at once, one handle per stream -- several decoders on one RNNLM (the paper's Section 3.1
 * has one search; a server has many).  Costs max_B * (6 H + 2 KB) bytes of device memory, not
 * another copy of the weights.  max_B: as in rnnlm_load, for calls through the new handle.
 * Release it with rnnlm_free.  Synchronous.
 */
int rnnlm_model_share(const rnnlm_model *model, int max_B, rnnlm_model **out);

/* Set a tunable (see rnnlm_option).  Host-side only; affects later calls. */
int rnnlm_set_option(rnnlm_model *model, int option, int value);

/* Wait for `hip_stream`, then return and clear the sticky rnnlm_device_flag bits in
 * *flags.  Returns a status. */
int rnnlm_last_error(rnnlm_model *model, void *hip_stream, int *flags);

/* Bytes of device workspace rnnlm_dedup / rnnlm_step_dedup need for N raw queries
 * (returns 0 for N <= 0).  The workspace must be 16-byte aligned. */
size_t rnnlm_dedup_workspace_bytes(int N);

/*
 * Group identical history ids (the cache lookup of Table 1, steps 1-3, for a whole batch:
 * a history seen before is not computed again; new ones are numbered in order of first
 * appearance, step 10).
 *   history_ids  dev u64[N]   any 64-bit value is an ordinary key (Section 3.2 packs a
 *                             context index and a small-LM index into one number).
 *   rep          dev i32[N]   out: rep[u] = smallest n holding the u-th distinct id;
 *                             ascending; only the first *n_unique entries are written.
 *   inverse      dev i32[N]   out: inverse[n] = u such that history_ids[rep[u]] == history_ids[n].
 *   n_unique     dev i32[1]   out: number of distinct ids.
 * The result is unique, hence bit-exact and run-to-run deterministic.  N = 0 writes
 * *n_unique = 0.  workspace: dev, rnnlm_dedup_workspace_bytes(N) bytes, contents undefined
 * before and after.
 */
int rnnlm_dedup(const uint64_t *history_ids, int N, int32_t *rep, int32_t *inverse,
                int32_t *n_unique, void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * rnnlm_dedup for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results
 * as rnnlm_dedup without `workspace`; the table lives in a fixed device array inside the library
 * (2.3 MB per GPU, held until the process ends), so N may not exceed RNNLM_DEDUP_STATIC_MAX_N
 * (RNNLM_ERANGE otherwise).  Calls no hipMalloc / hipFree, asynchronous on `hip_stream`.  All calls
 * on one GPU share the one array: calls that overlap in time on the same GPU (two streams, two
 * threads) race; order them.  The array's address is looked up on the first call on a device (or by
 * rnnlm_load / rnnlm_hs_load before that).
 */
#define RNNLM_DEDUP_STATIC_MAX_N 65536
int rnnlm_dedup_static(const uint64_t *history_ids, int N, int32_t *rep, int32_t *inverse,
                       int32_t *n_unique, void *hip_stream);

/*
 * Score one step for B distinct histories and N raw queries (ComputeRnnlm of Table 1,
 * step 6, batched):
 *   h_out[b][j]   = sigmoid(U[prev_word[b]][j] + sum_i W[j][i] h_in[b][i])
 *   logprob[n][k] = z_r[query_word[n][k]] - log sum_v exp z_r[v],   r = row_of_query[n],
 *                   z_r[v] = bias[v] + sum_j O[j][v] h_out[r][j]
 *   prev_word     dev i32[B]
 *   h_in          dev f32[B][H]   any finite values; all-zero rows are the utterance start
 *   query_word    dev i32[N][K]
 *   row_of_query  dev i32[N] with values in [0,B), or NULL meaning N == B and row n
 *   h_out         dev f32[B][H]   out; its B*H floats must not overlap those of h_in (RNNLM_EINVAL)
 *   logprob       dev f32[N][K]   out
 * The B x V logits never leave the chip; only N x K floats are written besides h_out.
 * B = 0 or N = 0 or K = 0 is a valid no-op for the corresponding outputs.
 */
int rnnlm_step(const rnnlm_model *model, int B, int K,
               const int32_t *prev_word, const float *h_in,
               const int32_t *query_word, const int32_t *row_of_query_or_null, int N,
               float *h_out, float *logprob, void *hip_stream);

/*
 * The whole path in one call, with no host round trip between grouping and scoring
 * (RnnlmProb of Table 1 for N (history, words) lookups at once): rnnlm_dedup on
 * history_ids, then rnnlm_step on the distinct histories only, each taken from its first
 * occurrence, with every raw query answered from its group's row.
 *   history_ids   dev u64[N]
 *   prev_word     dev i32[N]      per RAW query (equal ids must carry equal histories)
 *   h_in          dev f32[N][H]   per RAW query
 *   query_word    dev i32[N][K]
 *   rep, inverse, n_unique        out, as rnnlm_dedup
 *   h_out         dev f32[N][H]   out: row u < *n_unique = updated hidden vector of the
 *                                 u-th distinct history; rows beyond are left untouched
 *   logprob       dev f32[N][K]   out
 * Requires N <= max_B.  Either kind of model (full softmax or hierarchical output layer).
 */
int rnnlm_step_dedup(const rnnlm_model *model, int N, int K,
                     const uint64_t *history_ids, const int32_t *prev_word, const float *h_in,
                     const int32_t *query_word,
                     int32_t *rep, int32_t *inverse, int32_t *n_unique,
                     float *h_out, float *logprob,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ---- Cache kept between steps (Table 1 as a whole; Sections 4.2 and 5.3) ----------------
 *
 * rnnlm_step_dedup forgets everything when it returns.  The paper's Cache lives for an
 * utterance (or longer, within a size boundary): a history that was computed in an earlier
 * step is looked up, not computed again.  An rnnlm_cache keeps, on the device, for up to
 * `capacity` history ids the updated hidden vector and the normaliser of that history.
 * Nothing is ever removed: when it is full, further new histories are computed and answered
 * but not kept (Section 5.3 bounds the size and leaves a removal policy open).
 */
typedef struct rnnlm_cache rnnlm_cache;   /* opaque, owned by the library */

/* Create an empty cache for `model` (calls may pass up to the model's max_B queries).
 * capacity >= 0 entries; device memory ~ capacity * (4 H + 36) bytes.  Synchronous. */
int rnnlm_cache_create(const rnnlm_model *model, int capacity, rnnlm_cache **out);

/* Release a cache.  NULL is a no-op.  Synchronises the device. */
int rnnlm_cache_free(rnnlm_cache *cache);

/* Forget every entry and zero the counters (start of an utterance, Section 4.2).
 * Asynchronous on `hip_stream`. */
int rnnlm_cache_reset(rnnlm_cache *cache, void *hip_stream);

/* Wait for `hip_stream`, then write to the HOST array out[5]: entries held, and the running
 * totals over distinct histories per step: looked up, found, computed, computed but not
 * kept because the cache was full. */
int rnnlm_cache_stats(rnnlm_cache *cache, void *hip_stream, int64_t out[5]);

/*
 * rnnlm_step_dedup through the cache: the distinct histories of this call that the cache
 * holds take their stored hidden vector and normaliser (whatever prev_word / h_in say now);
 * only the others are computed, and they are stored, in order of first appearance, while
 * there is room.  Arguments as rnnlm_step_dedup, plus
 *   cache        the cache, or NULL for none (then exactly rnnlm_step_dedup)
 *   base_score   dev f32[N][K] or NULL: subtracted from the log-probabilities, so that the
 *                value that leaves the device is the difference to the short-span n-gram
 *                score the search already applied (Section 4.2, last paragraph)
 *   score        dev f32[N][K] out: logprob - base_score
 *   step_stats   dev i32[4] out or NULL: distinct histories, found in the cache, computed,
 *                entries held afterwards
 * h_out rows of histories found in the cache are copies of the stored vectors.  A stored
 * value is returned bit for bit as it was first computed.  Calls that share a cache must be
 * ordered on one stream.  Requires N <= max_B of the model the cache was created for.
 */
int rnnlm_step_cached(const rnnlm_model *model, rnnlm_cache *cache_or_null, int N, int K,
                      const uint64_t *history_ids, const int32_t *prev_word, const float *h_in,
                      const int32_t *query_word, const float *base_score_or_null,
                      int32_t *rep, int32_t *inverse, int32_t *n_unique,
                      float *h_out, float *score, int32_t *step_stats_or_null,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * ---- Hierarchical output layer (Section 2.1) ----------------------------------------------
 *
 * The paper's own output layer: the words are the leaves of a Huffman tree and the probability
 * of a word is normalised only over the nodes on its path from the root,
 *     log p(w | h') = sum over the path nodes i of log sigmoid(+-theta_i . h'),
 * + for code bit 0, - for code bit 1: about log2 V dot products per queried word, no
 * whole-vocabulary normalisation.  A model loaded with rnnlm_hs_load is stepped with
 * rnnlm_hs_step on rows the caller has made distinct (rnnlm_step refuses it, and rnnlm_hs_step a
 * full-softmax model), or, like any model, with rnnlm_step_dedup / rnnlm_step_cached on raw
 * queries: grouping of the history ids, the cache of Table 1 -- which for such a model keeps the
 * hidden vector of a history and nothing else, a path needs no normaliser -- and the paths of
 * the queried words in one call.  That is the paper's RnnlmProb as a whole: its cache around
 * its own output layer.
 */

/* Huffman tree over V >= 2 words from their frequencies (HOST arrays, host code): the path of
 * word v from the root down is path_entry[path_offset[v] .. path_offset[v+1]), each entry =
 * inner node (0 .. V-2, numbered in order of creation, the root is V-2) | code bit << 31.
 * Two-queue construction; of two equal weights a word goes before an inner node, words of
 * equal frequency in order of their id; the first of a merged pair gets code bit 0.
 *   path_offset  out i32[V+1]
 *   path_entry   out i32[capacity], may be NULL to ask for the size only
 *   needed       out, may be NULL: number of entries
 * Returns RNNLM_ERANGE (offsets and *needed valid) when capacity is too small. */
int rnnlm_huffman_build(int V, const double *frequency, int32_t *path_offset, int32_t *path_entry,
                        size_t capacity, size_t *needed);

/* Load a model with the hierarchical output layer.  U, W, dtype, max_B as rnnlm_load;
 *   Theta        [V-1][H]  vector of every inner node, same element type as U and W
 *   path_offset  i32[V+1], path_entry i32[path_offset[V]]  the tree, as rnnlm_huffman_build
 *                writes it (checked: non-empty paths, node ids below V-1)
 * All HOST pointers.  Synchronous. */
int rnnlm_hs_load(int V, int H, int dtype, const void *U, const void *W, const void *Theta,
                  const int32_t *path_offset, const int32_t *path_entry, int max_B, rnnlm_model **out);

/* rnnlm_step with the hierarchical output layer; arguments as rnnlm_step, plus base_score
 * (dev f32[N][K] or NULL) as in rnnlm_step_cached. */
int rnnlm_hs_step(const rnnlm_model *model, int B, int K, const int32_t *prev_word, const float *h_in,
                  const int32_t *query_word, const int32_t *row_of_query_or_null, int N,
                  const float *base_score_or_null, float *h_out, float *logprob, void *hip_stream);

/*
 * ---- IndexTable and its inverse on the device (Section 3.2; Table 1 steps 5 and 7-12) -------
 *
 * A context -- the word it ends in and its hidden vector (Section 4.1) -- is stored once and
 * stands for a 4-byte index from then on (Table 3), so a search that keeps only indices needs
 * no host-side id management: rnnlm_index_intern turns contexts given by value into indices
 * (the same context, compared word for word and bit for bit, always gets the same index; new
 * ones are numbered in order of first appearance), rnnlm_index_fetch gives the stored contexts
 * back.  Packed with the small-LM index by rnnlm_pack_ids, the indices are the history ids of
 * rnnlm_step_dedup / rnnlm_step_cached.
 */
typedef struct rnnlm_index_table rnnlm_index_table;   /* opaque, owned by the library */

enum {
    RNNLM_INDEX_NOT_STORED = 0xFFFFFFFFu,  /* the table was full: the context was not stored */
    RNNLM_INDEX_COLLISION  = 0xFFFFFFFEu   /* contents differ although the 64-bit hashes agree */
};

/* Create an empty table for hidden vectors of H floats, up to `capacity` contexts, calls of up
 * to max_N contexts.  Device memory ~ capacity * (4 H + 20) + 40 max_N bytes.  Synchronous. */
int rnnlm_index_create(int H, int capacity, int max_N, rnnlm_index_table **out);

/* Release a table.  NULL is a no-op.  Synchronises the device. */
int rnnlm_index_free(rnnlm_index_table *table);

/* Forget every context and zero the counters.  Asynchronous on `hip_stream`. */
int rnnlm_index_reset(rnnlm_index_table *table, void *hip_stream);

/*
 * Indices of N contexts given by value (inverse IndexTable, then IndexTable for the new ones).
 *   word   dev i32[N]     the word each context ends in
 *   h      dev f32[N][H]  its hidden vector
 *   index  dev u32[N]     out: the index; RNNLM_INDEX_NOT_STORED when the table was full;
 *                         RNNLM_INDEX_COLLISION when a different context with the same
 *                         64-bit hash is held (probability about 2^-64 per pair of contexts;
 *                         counted in rnnlm_index_stats)
 * Asynchronous on `hip_stream`; calls on one table must be ordered on one stream.
 */
int rnnlm_index_intern(rnnlm_index_table *table, int N, const int32_t *word, const float *h,
                       uint32_t *index, void *hip_stream);

/* The stored context of each index (IndexTable[c], Table 1 step 5): word dev i32[N] and
 * h dev f32[N][H], out.  An index the table does not hold gives word -1 and a NaN vector and is
 * counted in rnnlm_index_stats.  Asynchronous on `hip_stream`. */
int rnnlm_index_fetch(const rnnlm_index_table *table, int N, const uint32_t *index, int32_t *word,
                      float *h, void *hip_stream);

/* Wait for `hip_stream`, then write to the HOST array out[6]: contexts held, and running
 * totals: distinct contexts looked up per call, found, not stored because full, hash
 * collisions, bad indices passed to rnnlm_index_fetch. */
int rnnlm_index_stats(rnnlm_index_table *table, void *hip_stream, int64_t out[6]);

/*
 * The packed 8-byte index of Section 3.2: ids[n] = ctx_idx[n] << 32 | small_lm_idx[n]
 * (RNNLM context index in the high half, index of the graph-building LM in the low half).
 * All device pointers; asynchronous on `hip_stream`.
 */
int rnnlm_pack_ids(const uint32_t *ctx_idx, const uint32_t *small_lm_idx, int N, uint64_t *ids,
                   void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RNNLM_H_ */
