/*
 * confspec_generate.h - one generation step (Algorithm 1: the generate calls of the small and the large model) and
 * the full-vocabulary reading of the confidence (Section 4.2, the sentence after Eq. 3, read without restricting the
 * softmax to the verdict tokens).
 *
 * A generation step is the same pass as verification - the new tokens of every trace on top of its cached context -
 * followed by the language-model head over the whole vocabulary at the last position instead of the verdict rows
 * only.  With one new token per trace and write-back of its keys / values it is a decode step; with the drafted or
 * accepted tokens as suffix it is what produces the first token of the next step.
 *
 * A step with one new token in each of at most 32 traces of a bf16 model runs on kernels of its own (each weight
 * matrix streamed once against the activation rows, attention with one query row per head, the head fused with a
 * running arg max / log-sum-exp so that the [B, vocab] logits are never stored); every other batch takes the
 * verification pass's kernels and stores the logits in the head scratch.  confspec_tune "decode_kernels" = 0 switches
 * the former off.
 */
#ifndef CONFSPEC_GENERATE_H
#define CONFSPEC_GENERATE_H

#include "confspec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Outputs, dev, one entry per trace.  z = W_lm . RMSNorm(x_last) over the whole vocabulary. */
typedef struct {
    int32_t *token;    /* [B] arg max of z (lowest index on ties): the greedy next token                       */
    float *max_logit;  /* [B] z[token]                                                                          */
    float *lse;        /* [B] log sum_v exp z_v; the full-softmax probability of any token v is exp(z_v - lse)  */
    float *conf_full;  /* [B] largest full-vocabulary probability among the verdict tokens; NULL when no verdict
                              ids are given                                                                      */
} confspec_head_out;

/* Bytes of dev scratch the head needs for up to max_B traces (the [B, vocab] fp32 logits of the general path dominate). */
size_t confspec_head_scratch_bytes(const confspec_ctx *ctx, int32_t max_B);

/* The pass of confspec_verify on `batch`, then the full-vocabulary head at the last suffix position of every trace.
 *   dev_n_append / h_n_append : both NULL, or as in confspec_verify_append (kv pages are then written)
 *   h_verdict_ids, n_verdict  : NULL / 0, or verdict tokens for conf_full (as in confspec_verify)
 *   dev_workspace             : as in confspec_verify
 *   dev_head_scratch          : dev, 256-byte aligned, >= confspec_head_scratch_bytes(ctx, B)
 * Needs vocab % 128 == 0 for a bf16 model (vocab % 64 == 0 for fp32).  Never synchronises; allocates nothing.
 * The logits are computed from the final norm carried as two bf16 terms against the bf16 head with fp32
 * accumulation.  Errors as in confspec.h. */
int confspec_generate_step(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_n_append, const int32_t *h_n_append,
                           const int32_t *h_verdict_ids, int32_t n_verdict, void *dev_workspace, size_t workspace_bytes,
                           void *dev_head_scratch, size_t head_scratch_bytes, const confspec_head_out *out,
                           confspec_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_GENERATE_H */
