/*
 * confspec_append.h - the verification pass with write-back of accepted draft tokens into the paged cache
 * (Algorithm 1, Stage 3; Section 4.2, "Stage 3: Context Management and Fallback": the accepted draft steps join
 * the context).
 *
 * The suffix of a trace starts with the drafted step.  When (some of) its tokens are to join the context, their
 * keys and values are the ones the verification pass computes anyway; this entry point stores them instead of
 * dropping them.  Run on plain context chunks (n_append[b] = S_b) it is chunked prefill: a context cache can be
 * produced by this library's own kernels.
 */
#ifndef CONFSPEC_APPEND_H
#define CONFSPEC_APPEND_H

#include "confspec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* confspec_verify (same arguments, same outputs, bit for bit) that also writes, for every layer, trace b and
 * i < n_append[b], the key (rotated to position L_b + i) and the value of suffix token i into logical row L_b + i
 * of trace b: physical block block_table[b][(L_b + i) / block_size], slot (L_b + i) % block_size.
 *   dev_n_append : dev int32 [B]; h_n_append: the same values on the host.  0 <= n_append[b] <= S_b and
 *                  L_b + n_append[b] <= max_blocks_per_seq * block_size.
 *   kv           : k_pages / v_pages are WRITTEN here (everything else in this library only reads them); the block
 *                  table must already name a block for every row written.
 * The caller guarantees that no row written is a visible row (below L_b') of any trace b' of this batch, and that no
 * two traces write the same physical row; then the verdict outputs do not depend on the write-back.  prefix_lens
 * is not changed: the new rows become visible when the caller passes larger lengths in a later call.
 * Errors as confspec_verify; counts out of range give CONFSPEC_E_OUT_OF_RANGE before any launch. */
int confspec_verify_append(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_n_append, const int32_t *h_n_append,
                           const int32_t *h_verdict_ids, int32_t n_verdict, const float *h_tau, int32_t n_tau,
                           void *dev_workspace, size_t workspace_bytes, float *dev_verdict_logits, float *dev_conf,
                           int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_APPEND_H */
