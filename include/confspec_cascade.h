/*
 * confspec_cascade.h - the two-tier cascade over the drafted steps of a batch of requests
 * (Section 4.2, "Cascaded Decision Rule", Eq. 4; Algorithm 1, Stage 2).
 *
 * Every trace of the batch is one drafted step of one request (context + drafted step + target step +
 * verification prompt as suffix).  The small model verifies every trace; a decision whose confidence
 * reaches gamma is kept, the others are escalated to the large model (Eq. 4); within a request the
 * steps are then walked in order and accepted until the first rejection (the loop of Stage 2), which
 * gives m, the number of drafted steps that join the context (Stage 3).
 *
 * Tree-structured drafting (Section 4.3, Eq. 5): with a parent array the traces of a request form a tree of candidate
 * steps.  Cascaded verification is applied to every candidate; layer by layer, among the candidates that continue
 * the step chosen so far and pass, the one with the highest confidence (the small model's where its decision was
 * kept, the large model's where it was consulted; lowest index on ties) is chosen, until nothing passes.
 *
 * Both models read the same token ids (one tokenizer; the embedding tables may be padded to different
 * sizes, ids must be valid for both) and have each their own paged cache of the same contexts.  The large model's pass runs on the compacted sub-batch of the traces that can be consulted:
 * confidence below gamma and no earlier step of the request rejected by a confident small-model decision
 * (steps after such a rejection are never reached by the loop, so leaving them out changes nothing).
 *
 * Unlike confspec_verify this call synchronises the stream once, between the two passes: the size of the
 * second pass is decided on the device and the host plans its launches from it.
 */
#ifndef CONFSPEC_CASCADE_H
#define CONFSPEC_CASCADE_H

#include "confspec.h"

#ifdef __cplusplus
extern "C" {
#endif

#define CONFSPEC_NOT_REACHED (-1)

/* Requests: traces req_start[r] .. req_start[r+1]-1 are the drafted steps of request r, in order.
 * req_start[0] = 0, req_start[n_requests] = B, every request has at least one step.
 * req_start is a dev array, h_req_start a host copy with the same values. */
typedef struct {
    int32_t n_requests;
    const int32_t *req_start;
    const int32_t *h_req_start;
    /* Candidate trees, or both NULL for chains (step j continues step j-1): parent[b] = the trace that candidate b
     * continues, an earlier trace of the same request, or -1 for a candidate that continues the context itself.
     * dev int32 [B] and a host copy. */
    const int32_t *parent;
    const int32_t *h_parent;
} confspec_requests;

/* Outputs, all dev, written by the call.  verdict values are indices into the verdict id list;
 * index 0 is "accept". */
typedef struct {
    float *conf_draft;        /* [B]  confidence of the small model's decision                          */
    int32_t *verdict_draft;   /* [B]  the small model's decision                                        */
    float *conf_target;       /* [B]  the large model's confidence, NaN where its pass left the trace out */
    int32_t *verdict_target;  /* [B]  its decision, CONFSPEC_NOT_REACHED where left out                  */
    int32_t *decision;        /* [B]  cascaded decision of the steps the walk reaches (a chain: the accepted ones
                                      and the first rejection; a tree: every candidate that continues a chosen
                                      step or the context), CONFSPEC_NOT_REACHED elsewhere                */
    uint8_t *escalated;       /* [B]  1 where the loop consulted the large model                        */
    uint8_t *target_ran;      /* [B]  1 where the large model's pass included the trace                 */
    int32_t *accepted_steps;  /* [n_requests]  m = number of chosen steps                               */
    uint8_t *selected;        /* [B]  1 on the chosen steps (a chain: the first m); may be NULL         */
    float *conf_used;         /* [B]  the confidence that entered the selection (kept: the small model's,
                                      escalated: the large model's), NaN where not reached; may be NULL */
} confspec_cascade_out;

/* Bytes of dev scratch confspec_cascade needs for batches up to max_B traces and max_T suffix tokens with a
 * large-model block table of max_blocks_per_seq_target entries per trace. */
size_t confspec_cascade_scratch_bytes(int32_t max_B, int32_t max_T, int32_t max_blocks_per_seq_target);

/* One cascade over `batch`.  draft / target: contexts, packed weights, caches and workspaces (each sized by
 * confspec_workspace_bytes of its context for the whole batch) of the two models; verdict ids must lie inside both
 * vocabularies.  gamma in [0, 1] (values above 1 are allowed and escalate everything).  dev_scratch: 256-byte
 * aligned, >= confspec_cascade_scratch_bytes.  h_n_target (host, may be NULL) receives the number of traces in
 * the large model's pass.  Errors as in confspec.h, reported on the draft context; the checks of the
 * request list, the scratch, both caches and both workspaces happen before the first launch. */
int confspec_cascade(confspec_ctx *draft, const confspec_weights *draft_weights, const confspec_kv *draft_kv,
                     void *draft_workspace, size_t draft_workspace_bytes, confspec_ctx *target,
                     const confspec_weights *target_weights, const confspec_kv *target_kv, void *target_workspace,
                     size_t target_workspace_bytes, const confspec_batch *batch, const confspec_requests *requests,
                     const int32_t *h_verdict_ids, int32_t n_verdict, float gamma, void *dev_scratch,
                     size_t scratch_bytes, const confspec_cascade_out *out, int32_t *h_n_target,
                     confspec_stream stream);

/* The verification pass for candidates that share their context (Section 4.3: the W candidates of one step of
 * tree-structured drafting are verified in parallel on top of the same chain of thought).  Same inputs and outputs
 * as confspec_verify plus a partition of the batch into groups of consecutive traces:
 *   group_start  : dev int32 [n_groups + 1], h_group_start a host copy; group_start[0] = 0,
 *                  group_start[n_groups] = B, strictly increasing.
 * The traces of a group must have the same prefix length, and their block-table rows must name the same pages
 * (the kernels read the context of the whole group through the row of its first trace).  Attention then lays the
 * query rows of all candidates of a group side by side in its row tiles, so that every context chunk is staged
 * once per 128 rows of the group rather than once per 128 rows of each candidate; the suffix keys stay per
 * candidate (a row sees its own trace's tokens only).  Results equal those of confspec_verify on the same batch up
 * to the rounding differences of differently cut attention pieces.  Groups of one trace are the plain pass.
 * Errors: as confspec_verify; CONFSPEC_E_OUT_OF_RANGE for a malformed partition or unequal prefix lengths inside
 * a group. */
int confspec_verify_shared(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_group_start, const int32_t *h_group_start,
                           int32_t n_groups, const int32_t *h_verdict_ids, int32_t n_verdict, const float *h_tau,
                           int32_t n_tau, void *dev_workspace, size_t workspace_bytes, float *dev_verdict_logits,
                           float *dev_conf, int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_CASCADE_H */
