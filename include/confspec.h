/*
 * confspec.h - C ABI of the batched verification pass for confidence-gated
 * cascaded step verification on one AMD MI355X (gfx950).
 *
 * For each of B reasoning traces the library prefills the S_b suffix tokens
 * (drafted step + target step + verification prompt) through a decoder-only
 * transformer on top of that trace's cached context KV (L_b tokens, paged),
 * reads the last-position logits of the verdict tokens only, turns them into a
 * softmax confidence and compares it with a threshold.  This is the verifier
 * call of the paper (Section 4.2: Eq. 2 decision, Eq. 3 confidence, Eq. 4
 * gate; Algorithm 1, the verification loop), batched over traces.
 *
 * Conventions
 *  - Every function returns CONFSPEC_OK (0) or a negative CONFSPEC_E_* code and
 *    never throws.  confspec_last_error() gives a message for the last failure
 *    on that context.
 *  - Pointers documented "dev" are device pointers owned by the caller and must
 *    stay valid until the stream work of the call has completed.  Pointers
 *    documented "host" are read before the call returns.
 *  - After confspec_create() the library allocates and frees no device memory:
 *    scratch comes from the caller's workspace.  Calls never synchronise the
 *    stream; outputs are valid once the caller has synchronised it.
 *  - The KV cache and the weights are read-only.  The suffix is never written
 *    back into the cache (only accepted draft steps join the context: Algorithm
 *    1, Stage 3), its keys and values live in the workspace.
 *  - All host-checkable validation happens before the first launch, so a failed
 *    call has no device side effects.
 */
#ifndef CONFSPEC_H
#define CONFSPEC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CONFSPEC_OK 0
#define CONFSPEC_E_INVALID_ARG (-1)   /* null pointer, size out of its documented range         */
#define CONFSPEC_E_UNSUPPORTED (-2)   /* a shape or dtype the kernels do not implement           */
#define CONFSPEC_E_WORKSPACE (-3)     /* workspace or destination buffer too small / misaligned  */
#define CONFSPEC_E_OUT_OF_RANGE (-4)  /* token id, verdict id, length or tau outside its range   */
#define CONFSPEC_E_HIP (-5)           /* a HIP runtime call failed                               */

#define CONFSPEC_DTYPE_FP32 0
#define CONFSPEC_DTYPE_BF16 1

#define CONFSPEC_MAX_VERDICT 8
#define CONFSPEC_MAX_TAU 8

typedef struct confspec_ctx confspec_ctx;

/* A HIP stream handle (hipStream_t) passed as an opaque pointer; NULL = the default stream. */
typedef void *confspec_stream;

/* Decoder shape.  Pre-norm blocks: RMSNorm, rotary positions in the half-split pairing
 * (i, i + head_dim/2), grouped-query attention (q head i reads kv head i / (n_q_heads/n_kv_heads)),
 * SwiGLU MLP, no biases.  dtype is the storage type of weights and KV pages. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_theta, rms_eps;
    int32_t dtype; /* CONFSPEC_DTYPE_* */
} confspec_model_cfg;

/* Weights, all dev, element type = cfg.dtype, row-major [out_features, in_features].
 *   embed, lm_head : [vocab, d_model] (lm_head may alias embed); final_norm: [d_model]
 *   attn_norm[l], mlp_norm[l] : [d_model]
 *   wqkv[l]      : [(n_q_heads + 2 n_kv_heads) * head_dim, d_model], rows = q heads, k heads, v heads
 *   wo[l]        : [d_model, n_q_heads * head_dim]
 *   w_gate_up[l] : [2 d_ffn, d_model]; packed == 0: rows 0..d_ffn-1 gate, d_ffn..2 d_ffn-1 up;
 *                  packed == 1: row order produced by confspec_pack_weights
 *   w_down[l]    : [d_model, d_ffn]
 * The six per-layer members are HOST arrays of n_layers dev pointers. */
typedef struct {
    const void *embed, *lm_head, *final_norm;
    const void *const *attn_norm;
    const void *const *wqkv;
    const void *const *wo;
    const void *const *mlp_norm;
    const void *const *w_gate_up;
    const void *const *w_down;
    int32_t packed;
    /* Filled by confspec_pack_weights, ignored (may be anything) when packed == 0: IEEE-half copies of
     * the four matrices of the first n_f16_layers layers (host arrays of n_layers dev pointers, entries
     * past n_f16_layers are NULL).  confspec_verify runs those layers' GEMMs on fp16 operands, which
     * carry three more mantissa bits than bf16 at the same cost; see confspec_tune "first_layers_f16". */
    int32_t n_f16_layers;
    const void *const *wqkv_perm;  /* bf16 models: wqkv with the row blocks of every head reordered for the
                                      projection kernel that applies the rotary embedding itself (all layers) */
    const void *const *wqkv_f16;   /* half copy of wqkv_perm */
    const void *const *wo_f16;
    const void *const *w_gate_up_f16;
    const void *const *w_down_f16;
} confspec_weights;

/* Paged context cache, dev, read-only, element type = cfg.dtype.
 *   k_pages, v_pages : [n_layers][n_blocks][n_kv_heads][block_size][head_dim]; keys are stored
 *                      already rotated to their absolute positions
 *   block_table      : int32 [B][max_blocks_per_seq]; logical row j of trace b lives in physical
 *                      block block_table[b][j / block_size], slot j % block_size.  Entries past
 *                      ceil(L_b / block_size) are ignored.  Traces may share physical blocks.
 * Every used block id must be in [0, n_blocks); ids are clamped to that range on the device, so a
 * bad table gives wrong numbers, never an out-of-bounds access. */
typedef struct {
    const void *k_pages, *v_pages;
    int32_t n_blocks, block_size;
    const int32_t *block_table;
    int32_t max_blocks_per_seq;
} confspec_kv;

/* One batch of traces.  T = sum of suffix lengths; suffix tokens are packed trace after trace.
 *   suffix_ids  : dev int32 [T], each in [0, vocab) (clamped on the device)
 *   cu_suffix   : dev int32 [B+1], exclusive prefix sums of S_b (cu[0] = 0, cu[B] = T, S_b >= 1)
 *   prefix_lens : dev int32 [B], 0 <= L_b <= max_blocks_per_seq * block_size
 *   h_cu_suffix, h_prefix_lens : HOST copies of the two arrays above; they drive validation and
 *                 launch planning and must hold the same values as the device copies. */
typedef struct {
    int32_t B, T;
    const int32_t *suffix_ids;
    const int32_t *cu_suffix;
    const int32_t *prefix_lens;
    const int32_t *h_cu_suffix;
    const int32_t *h_prefix_lens;
} confspec_batch;

/* Creates a context for one model shape on HIP device `device`.
 * Supported: head_dim 64 or 128 for fp32; head_dim 128 for bf16; n_q_heads a multiple of
 * n_kv_heads; d_model, d_ffn and the projection widths multiples of 64.  Allocates a few KiB of
 * host memory only. */
int confspec_create(const confspec_model_cfg *cfg, int device, confspec_ctx **out);

/* Bytes of device workspace confspec_verify needs for any batch with T <= max_T, B <= max_B and
 * sum of prefix lengths <= max_sum_L. */
int confspec_workspace_bytes(const confspec_ctx *ctx, int32_t max_T, int32_t max_B, int64_t max_sum_L,
                             size_t *out_bytes);

/* Bytes of device memory confspec_pack_weights writes: all layers' reordered gate/up matrices and, for
 * a bf16 model, the reordered wqkv matrices and the fp16 copies of the first layers' matrices. */
int confspec_packed_bytes(const confspec_ctx *ctx, size_t *out_bytes);

/* One-time reordering of the gate/up rows so that one GEMM output tile holds a gate column and its
 * up column side by side (the SwiGLU product is then taken in the GEMM epilogue).  Reads in->w_gate_up
 * (packed == 0), writes dev_dst (256-byte aligned, >= confspec_packed_bytes), and fills *out with a
 * weights record whose w_gate_up pointers point into dev_dst and whose other members equal *in's.
 * For a bf16 model it also writes IEEE-half copies of the four matrices of the first layers (the number
 * confspec_verify would otherwise run with two-term activations), converted element by element: exact for
 * |w| >= 2^-14, rounded to the half subnormal grid (absolute error <= 2^-25) below that.
 * For a bf16 model it further writes, for every layer, a copy of wqkv whose rows are reordered inside each head
 * (blocks of 32 rows in the order 0, 2, 1, 3) for the projection kernel that rotates q and k in its epilogue.
 * h_ptr_storage: host array of 6 * n_layers pointers that the pointer-array members of *out set by this
 * call will point into; it must outlive *out.  Enqueued on `stream`. */
int confspec_pack_weights(confspec_ctx *ctx, const confspec_weights *in, void *dev_dst, size_t dst_bytes,
                          const void **h_ptr_storage, confspec_weights *out, confspec_stream stream);

/* The batched verification pass (Section 4.2, Eq. 2-4).
 *   w            : packed weights (w->packed == 1)
 *   h_verdict_ids: host int32 [n_verdict], 2 <= n_verdict <= CONFSPEC_MAX_VERDICT, distinct ids in
 *                  [0, vocab); by convention index 0 is the "accept the step" token
 *   h_tau        : host float [n_tau], 1 <= n_tau <= CONFSPEC_MAX_TAU, each in [0, 1]
 *   dev_workspace: dev, 256-byte aligned, >= confspec_workspace_bytes for this batch
 * Outputs (dev):
 *   dev_verdict_logits : float [B, n_verdict]  z_v = RMSNorm(x_last) . lm_head[verdict_ids[v]]
 *   dev_conf           : float [B]             softmax over the n_verdict logits, probability of the
 *                                              predicted decision (Eq. 3)
 *   dev_verdict        : int32 [B]             argmax index into verdict_ids (lowest index on ties)
 *   dev_accept         : uint8 [n_tau, B]      1 = conf >= tau: keep this model's decision;
 *                                              0 = escalate to the larger model (Eq. 4)
 */
int confspec_verify(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                    const confspec_batch *batch, const int32_t *h_verdict_ids, int32_t n_verdict,
                    const float *h_tau, int32_t n_tau, void *dev_workspace, size_t workspace_bytes,
                    float *dev_verdict_logits, float *dev_conf, int32_t *dev_verdict,
                    uint8_t *dev_accept, confspec_stream stream);

/* Message for the last error on this context ("" if none).  The pointer stays valid until the
 * next failing call on the context. */
const char *confspec_last_error(const confspec_ctx *ctx);

void confspec_destroy(confspec_ctx *ctx);

/* Library version, "major.minor". */
const char *confspec_version(void);

#ifdef __cplusplus
}
#endif
#endif /* CONFSPEC_H */
