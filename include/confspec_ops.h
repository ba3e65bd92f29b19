/*
 * confspec_ops.h - single-step entry points of the verification pass.
 *
 * confspec_verify() (confspec.h) is the product call.  The functions here run one step of it at a
 * time through the same kernels, so that each step can be checked and timed on its own: the
 * projection GEMMs with their epilogues, RMSNorm, the paged grouped-query attention, and the
 * verdict head with the confidence gate (Section 4.2, Eq. 3 and Eq. 4 of the paper for the last
 * one; the others are the decoder the verifier model runs on).  Same conventions as confspec.h:
 * dev pointers are caller-owned device memory, nothing is allocated, nothing synchronises.
 */
#ifndef CONFSPEC_OPS_H
#define CONFSPEC_OPS_H

#include "confspec.h"

#ifdef __cplusplus
extern "C" {
#endif

#define CONFSPEC_EPI_STORE_F32 0  /* out fp32 [M,N] = A . W^T                                   */
#define CONFSPEC_EPI_RESID_F32 1  /* out fp32 [M,N] += A . W^T (in place)                       */
#define CONFSPEC_EPI_SWIGLU 2     /* W rows gate/up interleaved (confspec_pack_weights order);   */
                                  /* out (model dtype) [M, N/2] = silu(gate) * up                */

/* Activation formats (bf16 contexts only beyond 1).  `a_terms` / `out_terms` are
 *   1  the context's dtype;
 *   2  two bf16 terms: an activation matrix [M, K] is carried as [M, 2K] = hi | lo, hi = bf16(v) and
 *      lo = bf16(v - hi), which keeps 16 mantissa bits through a bf16 MFMA GEMM at twice the k-loop length;
 *   3  IEEE half: 11 mantissa bits at the cost of a bf16 GEMM; in a GEMM both A and W then hold half values.
 * confspec_verify runs the first "split_layers" layers (see confspec_tune) in format 3 when the packed
 * weights carry half copies of those layers' matrices, else in format 2. */

/* C[M,N] = A[M,K] . W[N,K]^T with one of the epilogues above.  A ([M, a_terms*K]) and W are dev
 * arrays of the context's dtype (row-major, K contiguous).  Requires N % 128 == 0 and K % 64 == 0 for
 * bf16, N % 64 == 0 and K % 16 == 0 for fp32; any M >= 1.  out_terms != 1 is valid with the SwiGLU
 * epilogue only (2: out is [M, 2 * N/2]; 3: out holds half values).  dev_scratch (may be NULL) is dev memory the call may use for
 * partial products: with at least confspec_op_gemm_scratch_bytes() bytes a bf16 GEMM whose output has too few
 * 128 x 128 tiles to fill the chip, or whose k range is long (K >= 4096 elements) while 256 x 256 tiles cover only
 * a third to a sixth of the chip, cuts the k range into slices that run as separate workgroups and are added in
 * a fixed order; without it such a GEMM runs one workgroup per tile.  16-byte aligned. */
int confspec_op_gemm(confspec_ctx *ctx, const void *dev_A, const void *dev_W, void *dev_out, int32_t M,
                     int32_t N, int32_t K, int32_t epilogue, int32_t a_terms, int32_t out_terms,
                     void *dev_scratch, size_t scratch_bytes, confspec_stream stream);

/* Scratch bytes with which confspec_op_gemm takes its split-K path for this shape (0: it never does). */
size_t confspec_op_gemm_scratch_bytes(const confspec_ctx *ctx, int32_t M, int32_t N, int32_t K, int32_t a_terms);

/* out[t,:] = x[t,:] / sqrt(mean(x[t,:]^2) + rms_eps) * g, x fp32 [n_rows, d_model], g in the context's
 * dtype, out [n_rows, out_terms * d_model] in the context's dtype. */
int confspec_op_rmsnorm(confspec_ctx *ctx, const float *dev_x, const void *dev_g, void *dev_out,
                        int32_t n_rows, int32_t out_terms, confspec_stream stream);

/* Rotary embedding + split of a fp32 QKV projection [T, (Hq + 2 Hkv) hd] into q [T,Hq,hd],
 * k [T,Hkv,hd], v [T,Hkv,hd] (context dtype); positions are L_b + t from the batch.
 * dev_q_lo / dev_k_lo / dev_v_lo (bf16 contexts; all three or none, NULL = none) receive the second
 * bf16 term bf16(value - bf16(value)) in the same layouts. */
int confspec_op_rope_split(confspec_ctx *ctx, const confspec_batch *batch, int32_t max_prefix_len,
                           const float *dev_qkv, void *dev_q, void *dev_k, void *dev_v, void *dev_q_lo,
                           void *dev_k_lo, void *dev_v_lo, void *dev_workspace, size_t workspace_bytes,
                           confspec_stream stream);

/* QKV projection with the rotary embedding and the split in its epilogue (bf16 contexts, head_dim 128): the
 * same q, k, v (and second terms) as confspec_op_gemm into fp32 followed by confspec_op_rope_split, in one kernel.
 * dev_h: normalised activations [T, d_model] in activation format a_terms (1 bf16, 2 hi | lo, 3 half).
 * dev_wqkv_perm: wqkv with the 32-row blocks of every 128-row head in the order 0, 2, 1, 3 (what
 * confspec_pack_weights produces as wqkv_perm), bf16, or half values when a_terms == 3. */
int confspec_op_qkv_rope(confspec_ctx *ctx, const confspec_batch *batch, int32_t max_prefix_len, const void *dev_h,
                         int32_t a_terms, const void *dev_wqkv_perm, void *dev_q, void *dev_k, void *dev_v,
                         void *dev_q_lo, void *dev_k_lo, void *dev_v_lo, void *dev_workspace, size_t workspace_bytes,
                         confspec_stream stream);

/* Attention of one layer: softmax over keys j <= L_b + t of q . k_j / sqrt(hd), keys and values
 * 0..L_b-1 from the paged cache of `layer`, the rest from dev_k_suffix / dev_v_suffix.
 * q [T,Hq,hd], k/v suffix [T,Hkv,hd], out [T, out_terms*Hq*hd], all in the context's dtype.
 * With dev_q_lo / dev_k_lo / dev_v_lo given (bf16 contexts; all three or none) q and the suffix keys /
 * values are hi + lo two-term values and the kernel also carries its probabilities as two terms;
 * confspec_verify does this in the first "attn_precise_layers" layers. */
int confspec_op_attention(confspec_ctx *ctx, const confspec_kv *kv, const confspec_batch *batch, int32_t layer,
                          const void *dev_q, const void *dev_k_suffix, const void *dev_v_suffix, const void *dev_q_lo,
                          const void *dev_k_lo, const void *dev_v_lo, void *dev_out, int32_t out_terms,
                          void *dev_workspace, size_t workspace_bytes, confspec_stream stream);

/* Verdict head and gate on a residual stream x fp32 [T, d_model]: for each trace the last suffix
 * row is normalised, dotted with the verdict rows of lm_head, soft-maxed over the verdicts and
 * compared with every tau.  Outputs as in confspec_verify. */
int confspec_op_verdict_gate(confspec_ctx *ctx, const confspec_batch *batch, const float *dev_x,
                             const void *dev_final_norm, const void *dev_lm_head, const int32_t *h_verdict_ids,
                             int32_t n_verdict, const float *h_tau, int32_t n_tau, void *dev_workspace,
                             size_t workspace_bytes, float *dev_verdict_logits, float *dev_conf,
                             int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream);

/* The slices the pass carves its workspace into, in carving order: byte offsets and lengths (host arrays of *n
 * entries on entry, *n = number of slices on return, at most 48) and the total.  exact == NULL: the layout behind
 * confspec_workspace_bytes(T, B); otherwise the layout for that one batch (confspec_static_scratch_need).  For
 * checks of the layout on the host; nothing is launched. */
int confspec_op_workspace_slices(const confspec_ctx *ctx, int32_t T, int32_t B, const confspec_batch *exact,
                                 size_t *h_offsets, size_t *h_bytes, int32_t *n, size_t *total);

/* Phase timing of the pass, the library's profiling hook.  While it is switched on for a context, every
 * confspec_verify / confspec_verify_append / confspec_generate_step call on that context records a HIP event on
 * its stream wherever the pass moves from one phase to the next (a few hundred events per pass, created when the
 * timing is first switched on; they cost a few microseconds per pass).  confspec_phase_times waits for the last
 * event of the most recent call and returns, per phase, the summed time between its events in milliseconds and
 * (h_intervals, may be NULL) the number of intervals.  Do not capture a call into a HIP graph while timing is on. */
#define CONFSPEC_PHASE_NORM 0          /* stand-alone RMSNorm kernels                                               */
#define CONFSPEC_PHASE_QKV 1           /* QKV projection with rotary embedding and q / k / v split                  */
#define CONFSPEC_PHASE_ATTN 2          /* attention kernel, one-term variant, every layer it runs in                */
#define CONFSPEC_PHASE_ATTN_PRECISE 3  /* attention kernel, two-term variant of the first layer(s)                  */
#define CONFSPEC_PHASE_ATTN_MERGE 4    /* merge of the key-range pieces of split attention tiles                    */
#define CONFSPEC_PHASE_O_PROJ 5        /* output projection + residual (+ split-K reduce where split)               */
#define CONFSPEC_PHASE_GATE_UP 6       /* gate/up projection + SwiGLU                                               */
#define CONFSPEC_PHASE_DOWN 7          /* down projection + residual (+ reduce / next RMSNorm where split)          */
#define CONFSPEC_PHASE_OTHER 8         /* maps, plans, rotary table, embedding, gathers, cache write-back, heads    */
#define CONFSPEC_N_PHASES 9
#define CONFSPEC_PHASE_END 9           /* internal: closes the last interval                                        */
int confspec_phase_timing(confspec_ctx *ctx, int32_t enable);
int confspec_phase_times(confspec_ctx *ctx, float *h_ms /* [CONFSPEC_N_PHASES] */, int32_t *h_intervals);

/* Settings of one context (ctx != NULL), or the defaults that contexts created afterwards start from (ctx == NULL).
 * Nothing is process-wide at run time: two contexts in one process keep their own settings.  A setting that changes
 * the workspace or packed-weight size ("attn_target_items", "gemm_splitk", "split_layers", "first_layers_f16") must be
 * made before confspec_workspace_bytes / confspec_packed_bytes are asked; a call with too small a buffer fails with
 * CONFSPEC_E_WORKSPACE.
 *   "split_layers" (default -1 = the first half of the layers): number of leading layers in which confspec_verify
 *       carries the GEMM activations with more than 8 mantissa bits.
 *   "first_layers_f16" (default 1): those layers run on IEEE-half operands (read by confspec_pack_weights, which then
 *       makes the half copies, and by confspec_verify); 0: two bf16 terms against the bf16 weights.  Stores in the
 *       half format saturate at +-65504.
 *   "attn_precise_layers" (default 1): number of leading layers whose attention runs the two-term variant.
 *   "fuse_rope" (default 1): the QKV projection of a bf16 model applies the rotary embedding in its epilogue
 *       (0: projection to fp32, then a separate kernel).
 *   "prefetch_down" (default 1): while the gate/up projection of a bf16 layer runs, its workgroups also read the down
 *       projection's weights once, front to back, so that they sit in the last-level cache when the down projection's
 *       strided tile loads ask for them (given where the down projection runs one workgroup per tile; results are
 *       bit-identical with 0).
 *   "decode_kernels" (default 1): a bf16 pass with one new token in each of at most 32 traces (a generation step,
 *       Algorithm 1's generate calls) can run on kernels shaped for it - projections that stream each weight matrix once
 *       against the 32 activation rows, attention with one query row per head - when every layer's operands are single
 *       16-bit values and the scratch holds its partial results.  1: it does when d_model and the q width are at most
 *       1536 (where those kernels are the faster ones), 2: whenever the shapes allow, 0: never (such a pass then runs on
 *       the general kernels).
 *   "prune_last_layer" (default 1): in the last layer, attention rows, output projection and MLP are computed for the
 *       last position of each trace only (the only rows the verdict head reads; 0 computes every row).
 *   Launch shapes, for measurements: "gemm_tile" (0 heuristic; 1 = 128x128, 4 = 256x256, 7 = 192x96 workgroup tiles; a
 *       shape that does not divide N falls back to 128x128), "gemm_group_m" (0 heuristic, else tile rows per band of
 *       the GEMM's tile order), "gemm_splitk" (0 heuristic, 1..64 = split-K factor of every bf16 GEMM that is given
 *       scratch; 1 = never split), "gemm_short_tile" (default 1: split-K products of at most 32 rows use 32 x 128 tiles with
 *       four LDS stages; 0: 128 x 128 tiles with two), "attn_target_items" (concurrent workgroup slots assumed by the attention planner),
 *       "attn_min_chunks", "attn_split" (0 = planner's choice, 1..4 = equal key-range pieces with that split factor,
 *       5 = front-loaded pieces), "attn_kernel" (0 = the software-pipelined main loop, the register-staged one for
 *       items of fewer than 12 chunks on average; 1 = always the register-staged loop; 2 = always the pipelined one).
 * Returns CONFSPEC_E_INVALID_ARG for an unknown key or a value out of range. */
int confspec_tune(confspec_ctx *ctx, const char *key, int32_t value);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_OPS_H */
