/*
 * librnnlm -- measurement aids.  No part of the method (include/rnnlm.h holds that): these calls
 * time single kernels of it, for the benchmark and the profiles.  Same conventions as rnnlm.h.
 */
#ifndef RNNLM_DIAG_H_
#define RNNLM_DIAG_H_

#include "rnnlm.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Run only the output-projection + log-sum-exp kernel (the whole-vocabulary normalisation of
 * Section 2.1) on the hidden block left in the model by the latest step, `repeats` times back to
 * back on `hip_stream`, bracketed by HIP events on that stream, and return the mean time of one
 * launch in milliseconds in *ms_per_launch.  Synchronises the stream.
 *   B           rows the launch is sized for
 *   n_rows_dev  dev i32[1] or NULL: when given, the kernel reads the true number of rows (<= B)
 *               from it on the device, exactly as inside rnnlm_step_dedup / rnnlm_step_cached
 *               (where only the device knows the count); NULL launches as rnnlm_step does.
 */
int rnnlm_time_outproj(const rnnlm_model *model, int B, const int32_t *n_rows_dev_or_null, int repeats,
                       void *hip_stream, float *ms_per_launch);

/* Name (as a kernel trace shows it, without template arguments) of the kernel that a launch of the
 * output projection sized for B rows takes on this model with its current options; a static string,
 * NULL for a bad argument or a model with the hierarchical output layer. */
const char *rnnlm_outproj_kernel_name(const rnnlm_model *model, int B);

/* Only the path-evaluation kernel of rnnlm_hs_step (no hidden update) on
 * h_out as a step left it, `repeats` times back to back on `hip_stream` between HIP events on
 * that stream; mean time of one launch in milliseconds.  Synchronises the stream. */
int rnnlm_hs_time_query(const rnnlm_model *model, int B, int K, const int32_t *query_word,
                        const int32_t *row_of_query_or_null, int N, const float *h_out, float *logprob,
                        int repeats, void *hip_stream, float *ms_per_launch);

/*
 * What a kernel launch costs on this device whatever the kernel does: `repeats` (1..100000) launches
 * of an empty one-wave kernel back to back on `hip_stream` between two HIP events; mean time per
 * launch in MICROseconds.  The floor under every small kernel of a step (the grouping of ids, the
 * hidden update and the query gather of Table 1's RnnlmProb are such kernels).  Synchronises the stream.
 */
int rnnlm_time_empty_launch(int repeats, void *hip_stream, float *us_per_launch);

/*
 * The rate the bf16 matrix cores of the current device
 * sustain on a loop shaped like the output projection's inner loop (the whole-vocabulary
 * normalisation of Section 2 is where the time goes), so that the kernel's rate can be set against
 * what this device gives under load and not only against the data-sheet peak.  One workgroup of
 * eight waves per compute unit, chains of 32 dependent 32x32x16 bf16 MFMAs, no memory traffic.
 *   feed 0: both operands in registers; feed 1: one operand read from LDS four steps ahead and
 *           one exp2-and-add per produced logit in between (the output projection's steady state);
 *   data 0: all-zero operands; data 1: random bf16 of the size of weights and centred activations
 *           (the clock under matrix load depends on the data).
 * Runs `launches` (1..1000) launches back to back on the null stream between two HIP events,
 * synchronises, allocates and frees 0.6 MB of device memory of its own.  *tflops: dense bf16
 * TFLOP/s; *core_ghz (may be NULL): core clock during the last launch, from the kernel's own cycle
 * counter against the constant 100 MHz one.  RNNLM_EINVAL for arguments outside these ranges.
 */
int rnnlm_probe_mfma_rate(int feed, int data, int launches, double *tflops, double *core_ghz);

#ifdef __cplusplus
}
#endif
#endif /* RNNLM_DIAG_H_ */
