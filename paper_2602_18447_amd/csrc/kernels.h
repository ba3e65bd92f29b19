// Internal launch interface between the host API and the gfx950 kernels.
// Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include <hip/hip_fp16.h>
#include <stdint.h>
#include <atomic>
#include "attn_plan.h"

namespace cs {

typedef __hip_bfloat16 bf16;

// fp32 -> IEEE half, round to nearest even, saturating: a finite value beyond the half range becomes +-65504 rather
// than an infinity (one infinity in an activation would turn the residual stream, and with it the confidence, into
// NaN).  Every store of the fp16 activation format goes through this.
__device__ __forceinline__ __half to_half_sat(float v) {
    return __float2half_rn(__builtin_amdgcn_fmed3f(v, -65504.0f, 65504.0f));
}

// Launch-shape settings of one context (confspec_tune); the kernels' launchers and the planners take them as an
// argument, nothing here is process-wide.
struct GemmTune {
    int tile = 0;      // 0 = heuristic; 1 = 128x128, 4 = 256x256 / 8 wavefronts, 7 = 192x96 / 6 wavefronts
    int group_m = 0;   // 0 = heuristic; otherwise tile rows per band of the tile order
    int splitk = 0;    // 0 = heuristic; otherwise the split-K factor of every GEMM that has scratch (1 = never split)
    int short_tile = 1;   // 1 = split-K products of at most 32 rows use 32 x 128 tiles with four LDS stages
};
// hipFuncSetAttribute(MaxDynamicSharedMemorySize) once per device and kernel: `mask` holds one bit per device.
inline hipError_t set_dynamic_lds_once(std::atomic<uint32_t> &mask, const void *fn, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    const uint32_t bit = 1u << (dev & 31);
    if (mask.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    mask.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
}

// ---- attention work description and planner arithmetic: attn_plan.h ----

enum Epilogue : int { EPI_STORE_F32 = 0, EPI_RESID_F32 = 1, EPI_SWIGLU = 2, EPI_ROPE = 3 };

// EPI_ROPE (bf16 model, head_dim 128): the GEMM is the QKV projection with the rows of every head of W
// reordered [0..31, 64..95, 32..63, 96..127], so that a wavefront's 64 output columns hold 32 rotation pairs
// (i, i + 64).  The epilogue rotates q and k heads by the token's position and writes q, k and v in the natural
// head layout, in bf16; the *_lo buffers (all or none) receive bf16(value - bf16(value)).
struct RopeArgs {
    const float *cos_t, *sin_t;   // [M, 64]
    void *q, *k, *v;              // [M, Hq, 128], [M, Hkv, 128], [M, Hkv, 128]
    void *q_lo, *k_lo, *v_lo;
    int32_t Hq, Hkv;
};

// ---- small kernels (templated on storage type: float or bf16) ----
hipError_t launch_prep(const int32_t *cu, const int32_t *plens, int B, int T, int max_L,
                       int32_t *tok_trace, int32_t *tok_pos, int32_t *last_row, hipStream_t s);
hipError_t launch_rope_table(const int32_t *tok_pos, int T, int hd, float theta, float *cos_t, float *sin_t,
                             hipStream_t s);
hipError_t launch_embed(int dtype, const int32_t *ids, const void *E, float *x, int T, int d, int vocab,
                        hipStream_t s);
// x fp32 [T,d] -> out (storage dtype) [T, d]; terms == 2 (bf16 only): [T, 2d] hi | lo two-term form;
// terms == 3 (bf16 only): IEEE half values
hipError_t launch_rmsnorm(int dtype, const float *x, const void *g, void *out, int T, int d, float eps,
                          int terms, hipStream_t s);
// qkv fp32 [T, (Hq+2Hkv) hd] -> q [T,Hq,hd], ksuf [T,Hkv,hd], vsuf [T,Hkv,hd] (storage dtype), q and k rotated
// q_lo / k_lo / v_lo (bf16 only, all or none): receive bf16(value - bf16(value))
hipError_t launch_rope_split(int dtype, const float *qkv, const float *cos_t, const float *sin_t, void *q,
                             void *ksuf, void *vsuf, void *q_lo, void *k_lo, void *v_lo, int T, int Hq, int Hkv,
                             int hd, hipStream_t s);
// dst row b = src row rows[b] (rows == nullptr: row b), row_bytes a multiple of 16
hipError_t launch_gather_rows(const void *src, void *dst, const int32_t *rows, int n_rows, int n_src_rows,
                              size_t row_bytes, hipStream_t s);
hipError_t launch_bf16_to_f16(const void *src, void *dst, size_t n, hipStream_t s);
// dst rows = src rows with the two middle 32-row blocks of every 128-row head swapped (n_heads * 128 rows of d elements)
hipError_t launch_permute_heads(const void *src, void *dst, int n_heads, int d, hipStream_t s);
hipError_t launch_pack_gate_up(int dtype, const void *src, void *dst, int F, int d, hipStream_t s);

struct VerdictArgs {
    int32_t ids[8];
    float tau[8];
    int32_t n_verdict, n_tau;
};
// last_row == nullptr: trace b reads row b of x
hipError_t launch_verdict(int dtype, const float *x, const int32_t *last_row, const void *final_norm,
                          const void *lm_head, VerdictArgs va, int B, int T, int d, float eps, float *logits,
                          float *conf, int32_t *verdict, uint8_t *accept, hipStream_t s);

// Arg max / max / log-sum-exp of every row of logits [B, V]; conf_full (may be null) from verdict_logits [B, n_verdict].
hipError_t launch_head_reduce(const float *logits, int B, int V, const float *verdict_logits, int n_verdict, int32_t *token,
                              float *max_logit, float *lse, float *conf_full, hipStream_t s);

// ---- GEMM: C[M,N] = A[M,K] . W[N,K]^T with an epilogue ----
//  EPI_STORE_F32: out fp32 [M,N]
//  EPI_RESID_F32: out fp32 [M,N] += result (in place)
//  EPI_SWIGLU   : W rows are gate/up interleaved in groups of 32; out (storage dtype) [M, N/2]
hipError_t launch_gemm_f32(const float *A, const float *W, void *out, int M, int N, int K, int epi,
                           hipStream_t s);
// Activation formats (a_terms / out_terms): 1 = bf16; 2 = two bf16 terms, A is [M, 2K] = hi | lo and a
// SwiGLU result is written as [M, 2 * N/2] = hi | lo; 3 = fp16 (A and W hold IEEE half values, a SwiGLU
// result is written as fp16).
// splitk_ws (may be null): scratch for the split-K path that outputs with too few 128 x 128 tiles to fill the
// chip, and long k ranges over few 256 x 256 tiles, take (gemm_splitk_factor > 1); it needs
// gemm_splitk_bytes(M, N, K * a_terms) bytes, otherwise the call falls back to one workgroup per tile.
// pf (may be null; used by the SwiGLU epilogue's wide kernel only): memory the kernel reads once, front to back,
// while it works, so that it sits in the last-level cache for the kernel that follows; n16 = 16-byte vectors.
struct PrefetchArgs {
    const void *ptr = nullptr;
    unsigned n16 = 0;
};
// norm (may be null; residual epilogue only): the RMSNorm that follows the projection in the pass.  When the call takes
// the split-K path, the kernel that adds the slices to the residual stream also writes RMSNorm(updated row) * g to
// norm->h (format norm->terms) and *norm_done becomes true; otherwise the caller runs the RMSNorm kernel itself.
struct NormAfter {
    const void *g = nullptr;
    void *h = nullptr;
    float eps = 0.f;
    int terms = 1;
};
hipError_t launch_gemm_bf16(const GemmTune &tune, const bf16 *A, const bf16 *W, void *out, int M, int N, int K, int epi,
                            int a_terms, int out_terms, float *splitk_ws, size_t splitk_ws_bytes, hipStream_t s,
                            const PrefetchArgs *pf = nullptr, const NormAfter *norm = nullptr, bool *norm_done = nullptr);
hipError_t launch_gemm_bf16_rope(const GemmTune &tune, const bf16 *A, const bf16 *W_perm, int M, int N, int K, int a_terms,
                                 const RopeArgs &rope, float *splitk_ws, size_t splitk_ws_bytes, hipStream_t s);
int gemm_splitk_factor(const GemmTune &tune, int M, int N, int K_total, bool *big_tile = nullptr);   // *big_tile: slices of 256 x 256 tiles
size_t gemm_splitk_bytes(const GemmTune &tune, int M, int N, int K_total);
size_t gemm_splitk_max_bytes(const GemmTune &tune, int max_M, int N, int K_total);   // largest gemm_splitk_bytes over M <= max_M

// ---- attention ----
struct AttnArgs {
    const void *q;          // [T, Hq, hd]
    const void *ksuf;       // [T, Hkv, hd] suffix keys (rotated)
    const void *vsuf;       // [T, Hkv, hd]
    const void *q_lo;       // second bf16 terms of q / ksuf / vsuf (same layouts), or nullptr: when all
    const void *ksuf_lo;    // three are given the bf16 kernel runs its two-term variant (q, suffix k/v
    const void *vsuf_lo;    // and the probabilities each carried as hi + lo)
    const void *k_pages;    // this layer's pages [n_blocks, Hkv, bs, hd]
    const void *v_pages;
    const int32_t *block_table;  // [B, max_blocks]
    const int32_t *cu;           // [B+1]
    const int32_t *plens;        // [B]
    const int32_t *tok_trace;    // [T] trace of every packed suffix token (written by the prep kernel)
    void *out;              // [T, Hq*hd] in activation format out_terms: 1 storage dtype, 2 bf16 hi | lo
                            // ([T, 2*Hq*hd]), 3 IEEE half
    int32_t B, T, Hq, Hkv, hd, n_blocks, block_size, max_blocks;
    float scale;            // 1/sqrt(hd)
    int32_t out_terms;
};
hipError_t launch_attn_f32(const AttnArgs &a, const int32_t *tok_trace, const int32_t *tok_pos, hipStream_t s);

// group_start: null (every trace is its own context unit) or n_units + 1 trace indices, dev (attn_plan.h)
hipError_t launch_attn_plan(const int32_t *cu, const int32_t *plens, const int32_t *group_start, int n_units, int B,
                            int T, int max_L, int G, int Hkv, int chunks_per_item, int equalize, int last_only,
                            int max_tiles, int max_items, AttnTile *tiles, AttnItem *items,
                            int32_t *counts /*[11]: tiles, items, first item of XCD 0..8*/, hipStream_t s);
// The attention kernel over the planned items; pieces of split tiles leave fp32 partial results in part_o / part_ml.
// avg_chunks: average number of key chunks per item (chooses the main loop)
hipError_t launch_attn_bf16(const AttnTune &tune, const AttnArgs &a, const AttnItem *items, const int32_t *counts,
                            int n_items_host, int max_xcd_items, int avg_chunks, float *part_o, float *part_ml, hipStream_t s);
// Combines the partial results of every split tile in piece order and writes the output rows.
hipError_t launch_attn_merge(const AttnArgs &a, const AttnTile *tiles, const int32_t *counts, int n_tiles_host,
                             const float *part_o, const float *part_ml, hipStream_t s);

// Suffix keys / values [T, Hkv, hd] of the tokens i < n_append[b] of every trace into rows L_b + i of the paged cache
// of one layer (k_pages / v_pages point at that layer).
hipError_t launch_kv_append(const void *ksuf, const void *vsuf, void *k_pages, void *v_pages, const int32_t *table,
                            const int32_t *cu, const int32_t *plens, const int32_t *n_append, const int32_t *tok_trace,
                            int B, int T, int Hkv, size_t head_row_bytes, int block_size, int max_blocks, int n_blocks,
                            hipStream_t s);

// ---- generation steps: one new token per trace (decode_bf16.hip) ----
constexpr int DEC_MAX_ROWS = 32;     // traces of a step the decode-shaped kernels take
constexpr int DEC_PIECE = 256;       // keys per attention workgroup
constexpr int DEC_MAX_G = 8;         // q heads per kv head
constexpr int DEC_MAX_KT = 24;       // k-tiles (of 64) of one k slice of a projection: 96 KiB of activations in LDS
// control block (int32): the arrival counters
constexpr int DEC_CTL_ATTN = 0;                          // + trace * Hkv + kv head
constexpr int DEC_CTL_TILE = DEC_CTL_ATTN + 1024;        // + column group of a sliced projection (<= 256)
constexpr int DEC_CTL_INTS = DEC_CTL_TILE + 256;
enum DecEpilogue : int { DEC_EPI_ROPE = 0, DEC_EPI_RESID = 1, DEC_EPI_SWIGLU = 2, DEC_EPI_HEAD = 3 };

// One projection of a step: out = X[M, K] . W[N, K]^T, M <= 32, K % 64 == 0, N % 16 == 0, then the epilogue.
struct DecGemm {
    const bf16 *X;            // [M, ldx], bf16 or (f16 != 0) IEEE half
    // ssq_in != null (ROPE, SWIGLU): X holds x * g without the 1 / rms factor of the RMSNorm; ssq_in [ssq_n, 32] are
    // partial sums of squares of every row (left by the preceding residual projection), the result rows are scaled by
    // 1 / sqrt(sum / K + eps)
    const float *ssq_in;
    int32_t ssq_n;
    float eps;
    const bf16 *W;            // [N, K], same element type
    int32_t ldx, M, K;
    int32_t n_ct;             // 16-column tiles of the accumulator: N / 16 (ROPE, RESID), N / 16 = F / 8 (SWIGLU)
    int32_t S, nwg;           // k slices and workgroups per slice (dec_gemm_plan)
    float *planes;            // S > 1: [S, 32, 16 n_ct] fp32 partial products
    int32_t *tile_cnt;        // S > 1: nwg arrival counters (zero before and after the launch)
    // RESID: x [M, N] fp32 += product.  With xg_out (may be null) it also writes the operand of the projection that
    // follows, x * g_next in format xg_fmt (1 bf16, 3 half) [M, N], and ssq_out [N / 16, 32]: the sum of squares of
    // each 16 columns of every updated row.
    float *x;
    void *xg_out;
    const bf16 *g_next;
    float *ssq_out;
    int32_t xg_fmt;
    // SWIGLU: W rows are gate / up interleaved in groups of 32; act [M, F] in format act_fmt (1 or 3)
    void *act;
    int32_t act_fmt;
    // HEAD: X is [M, 2 K] two-term bf16 (hi | lo), W the [vocab, K] head; the logits are never stored: every workgroup
    // leaves (max, index of the first max, sum of exp(z - max)) of its columns per row in head_part [nwg, 32, 4] fp32
    float *head_part;
    // ROPE: the QKV projection; perm != 0: W rows of every head reordered [0..31 | 64..95 | 32..63 | 96..127].
    // q also leaves its second bf16 term in rope.q_lo when that is not null.  With n_append (dev, may be null) the new
    // key / value row of every trace b with n_append[b] > 0 is also written to row plens[b] of its paged cache.
    RopeArgs rope;
    int32_t perm;
    void *k_pages, *v_pages;  // this layer's pages
    const int32_t *table, *plens, *n_append;
    int32_t max_blocks, n_blocks;
};
void dec_gemm_plan(int K, int n_ct, int *S, int *nwg);
size_t dec_gemm_plane_bytes(int K, int n_ct);      // 0 when the projection needs no partial planes
hipError_t launch_dec_gemm(const DecGemm &a, int epi, bool f16, hipStream_t s);
// token / max logit / log-sum-exp (and conf_full, with verdict logits) of B rows from the nwg records per row
hipError_t launch_dec_head_final(const float *part, int nwg, int B, const float *verdict_logits, int n_verdict, int32_t *token,
                                 float *max_logit, float *lse, float *conf_full, hipStream_t s);

struct DecAttn {
    const bf16 *q, *q_lo;             // [B, Hq, 128]; q_lo may be null
    const bf16 *ksuf, *vsuf;          // [B, Hkv, 128]: key / value of the new token
    const bf16 *k_pages, *v_pages;    // this layer's pages [n_blocks, Hkv, 16, 128]
    const int32_t *table, *plens;
    int32_t *ctl;                     // control block (launch_dec_init)
    void *out;                        // [B, Hq * 128] in format out_fmt (1 bf16, 3 half; 2: [B, 2 Hq 128] hi | lo)
    float *part_o, *part_ml;          // per (trace, piece, kv head): [8, 128] and [8, 2] fp32; B * max_pieces * Hkv of them
    int32_t B, Hq, Hkv, G, max_blocks, n_blocks, max_L, out_fmt;
    int32_t n_iter;                   // rounds of DEC_PIECE keys per workgroup (dec_attn_rounds)
    int32_t max_pieces;               // pieces of the longest trace: max_L / (DEC_PIECE * n_iter) + 1
    float scale_log2;                 // log2(e) / sqrt(head_dim)
};
hipError_t launch_dec_init(int32_t *ctl, hipStream_t s);
int dec_attn_rounds(int B, int Hkv, int max_L);
hipError_t launch_dec_attn(const DecAttn &a, hipStream_t s);
inline size_t dec_attn_part_o_bytes(int64_t n_pieces, int Hkv) { return (size_t)n_pieces * Hkv * DEC_MAX_G * 128 * 4; }
inline size_t dec_attn_part_ml_bytes(int64_t n_pieces, int Hkv) { return (size_t)n_pieces * Hkv * DEC_MAX_G * 2 * 4; }

// ---- cascade (cascade.hip) ----
hipError_t launch_cascade_select(const uint8_t *keep, const int32_t *verdict_d, const int32_t *req_start, const int32_t *parent,
                                 int R, int B, const int32_t *cu, const int32_t *plens, int T, uint8_t *open_flag,
                                 uint8_t *target_ran, int32_t *pos_of, int32_t *sel_idx, int32_t *cu_out, int32_t *plens_out,
                                 int32_t *n_out, hipStream_t s);
hipError_t launch_cascade_gather(const int32_t *pos_of, const int32_t *cu, const int32_t *cu_out, const int32_t *ids,
                                 int32_t *ids_out, const int32_t *table, int32_t *table_out, int max_blocks, int B, int T,
                                 hipStream_t s);
hipError_t launch_cascade_merge(const uint8_t *keep, const int32_t *verdict_d, const float *conf_d, const int32_t *pos_of,
                                const float *conf_t_c, const int32_t *verdict_t_c, const int32_t *req_start,
                                const int32_t *parent, int R, int B, int n_target, float *conf_t, int32_t *verdict_t,
                                int32_t *decision, uint8_t *escalated, uint8_t *selected, float *conf_used, int32_t *accepted,
                                hipStream_t s);

}  // namespace cs
