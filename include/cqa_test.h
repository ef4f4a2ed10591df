/*
 * cqa_test.h -- test hooks and measurement helpers of libcqa.
 *
 * Not part of the product boundary (that is cqa.h): these calls exist so that the
 * parity tests can force kernel variants and split counts and read back what the
 * adaptive decode decided, and so that the benchmark can time individual kernels.
 * Same conventions as cqa.h (plain C, int32_t status, host / device pointers as
 * named).  All of them may wait for the device.
 */
#ifndef CQA_TEST_H
#define CQA_TEST_H

#include "cqa.h"

#ifdef __cplusplus
extern "C" {
#endif

/* ---- test hooks ------------------------------------------------------------ */

/* What the last adaptive decode decided, copied to the host after a
 * device synchronise.  k_star_host int32 [batch][n_q_heads]; selected_host int32
 * [batch][n_q_heads][512] (the head's own blocks, best first; entries past K*
 * are unspecified); promoted_host uint16 [batch][n_kv_heads][n_blocks] (bit 0 = some head
 * of the group scored this block with FP16 keys, bit 1 = some head attended its FP16 values,
 * bits 4-7 / 8-11 = which of the group's heads did, head i of the group at bit 4 + i / 8 + i);
 * logmass_int8_host / logmass_mixed_host float [batch][n_q_heads][n_blocks] (block
 * log-masses of step 1, and of step 4 where a block was revisited, else step 1's); v_count_host int32 [batch][n_q_heads] and
 * v_selected_host int32 [batch][n_q_heads][512] (the head's value selection, largest
 * contribution first); contrib_host float [batch][n_q_heads][n_blocks] (the estimated
 * contributions p_b eta_b the value selection ranked; valid when v_limit > 0);
 * score_dev_host float [batch][n_q_heads] (largest |s_fp16 - s_int8| the canary saw
 * on the head's key-promoted tokens; valid when sel->canary was set).
 * Any pointer may be NULL.  n_blocks = sealed blocks of `layer`. */
int32_t cqa_adaptive_state(cqa_cache* c, int32_t layer, int32_t* k_star_host,
                           int32_t* selected_host, uint16_t* promoted_host,
                           float* logmass_int8_host, float* logmass_mixed_host,
                           int32_t* v_count_host, int32_t* v_selected_host, float* contrib_host,
                           float* score_dev_host);

/* Overrides the automatic split count (0 restores it).  For tests. */
int32_t cqa_set_splits(cqa_cache* c, int32_t n_splits);

/* How the matrix-core decode kernel loads Tier-1 records: 0 = chosen from the bytes a
 * whole decode step (all layers) streams, the default; 1 = plain loads; 2 = loads with
 * the non-temporal hint.  Results do not depend on it.  For tests and measurement. */
int32_t cqa_set_stream_hint(cqa_cache* c, int32_t mode);

/* Chooses the split-K decode kernel: 0 = matrix-core (MFMA) kernel, the default;
 * 1 = the vector-ALU kernel (same results to rounding; kept as a cross-check). */
int32_t cqa_set_kernel_variant(cqa_cache* c, int32_t variant);

/* ---- measurement ----------------------------------------------------------- */

/* The streaming-read ceiling of the split pass: launches, `iters` times back to back,
 * a kernel that loads the Tier-1 records of `layer` with the split pass's launch
 * shape and load instructions and computes nothing, and returns its mean duration
 * (milliseconds, host) and the bytes one launch reads (host, may be NULL).  For
 * benchmarks: achieved bandwidth of the split pass / this = how much of what the
 * memory system delivers for this access pattern the pass reaches. */
int32_t cqa_time_stream_read(cqa_cache* c, int32_t layer, int32_t iters, float* ms_per_launch,
                             int64_t* bytes_per_launch, void* stream);

/* Launches cqa_certified_decode `iters` times back to back on `stream`,
 * bracketed by HIP events recorded on that same stream, synchronises, and
 * returns the mean duration of one step in milliseconds in *ms_per_step
 * (host).  For benchmarks; the outputs hold the last iteration's results. */
int32_t cqa_time_certified_decode(cqa_cache* c, int32_t layer, const void* q_fp16_dev,
                                  const cqa_tolerances* tol, float* O_dev,
                                  cqa_head_cert* cert_dev, uint32_t* flags_dev,
                                  float* blk_logmass_dev, int32_t iters, float* ms_per_step,
                                  void* stream);

/* Per-launch timing of the split-K decode kernel (the dominant kernel), taken
 * with HIP event pairs attached to its dispatch on the stream each
 * cqa_certified_decode / cqa_decode_step call launches it on (the pair brackets
 * the kernel's execution, not the launch overhead).  begin arms up to max_launches pairs
 * (<= 65536); end synchronises on them and returns the mean and minimum kernel
 * duration in milliseconds and the number of launches timed (host pointers,
 * any may be NULL).  For benchmarks. */
int32_t cqa_profile_begin(cqa_cache* c, int32_t max_launches);
int32_t cqa_profile_end(cqa_cache* c, float* mean_ms, float* min_ms, int32_t* n_launches);
/* The individual durations (milliseconds, launch order) of the launches timed by the last
 * cqa_profile_begin / cqa_profile_end pair: copies min(n_launches, cap) values to ms_host and
 * returns the number of launches in *n_launches (host, may be NULL).  Call after cqa_profile_end. */
int32_t cqa_profile_durations(cqa_cache* c, float* ms_host, int32_t cap, int32_t* n_launches);

#ifdef __cplusplus
}
#endif
#endif /* CQA_TEST_H */
