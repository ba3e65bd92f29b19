/*
 * confspec_static.h - the verification pass for callers that cannot allocate device memory.
 *
 * For code that runs under HIP graph capture, tight serving loops and harnesses that forbid hipMalloc: the same
 * pass as confspec_verify (confspec.h), with the workspace taken from an array that is part of the library's code
 * object instead of from the caller.  The call allocates and frees nothing, on the device or through any library.
 */
#ifndef CONFSPEC_STATIC_H
#define CONFSPEC_STATIC_H

#include "confspec.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Size of the library's own scratch array.  Every GPU the library runs on holds one copy from the time the
 * library is loaded there until the process ends. */
#define CONFSPEC_STATIC_SCRATCH_BYTES (64u << 20)

/* Scratch bytes this batch needs with this context's settings.  Unlike confspec_workspace_bytes, which bounds every
 * batch of up to T tokens in B traces, the figure is for this batch alone (the attention plan's lists and partial
 * results and the split-K planes sized by what its lengths need), computed from the host arrays of `batch`
 * (B, T, h_cu_suffix, h_prefix_lens; the dev pointers are not touched).  confspec_verify_static accepts the batch iff
 * it is <= CONFSPEC_STATIC_SCRATCH_BYTES.  Draft-shaped model (d_model 1536, d_ffn 8960): about 200 suffix tokens,
 * or a one-token-per-trace batch of 64 traces. */
int confspec_static_scratch_need(const confspec_ctx *ctx, const confspec_batch *batch, size_t *out_bytes);

/* confspec_verify without the workspace arguments: same inputs, same outputs, same kernels and launch shapes, bit-identical results.
 * Returns CONFSPEC_E_WORKSPACE, before anything is launched, when the batch needs more scratch than the array holds
 * (then use confspec_verify).  The calling thread's current device must be the context's.  All calls on one GPU
 * share that GPU's array and it keeps the last call's contents; the pass writes every part of it before reading
 * it, so nothing needs clearing, but two calls whose stream work overlaps in time on one GPU (different streams,
 * or different threads) race on it: serialise them, or use confspec_verify with separate workspaces. */
int confspec_verify_static(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *h_verdict_ids, int32_t n_verdict,
                           const float *h_tau, int32_t n_tau, float *dev_verdict_logits, float *dev_conf,
                           int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_STATIC_H */
