// Host side of the C ABI: argument validation, workspace carving and the launch sequence of the
// batched verification pass.  No device memory is allocated here; every check that can be made from
// host-visible arguments happens before the first launch.  confspec_verify, confspec_verify_append and
// confspec_generate_step never synchronise the stream; confspec_cascade synchronises it once (the
// large model's launches are planned from the number of escalated traces).
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/confspec.h"
#include "../../include/confspec_ops.h"
#include "../../include/confspec_cascade.h"
#include "../../include/confspec_append.h"
#include "../../include/confspec_generate.h"
#include "../../include/confspec_static.h"
#include "kernels.h"

// Scratch of confspec_verify_static: one array per GPU, part of the loaded code object, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; the device address it yields is what is passed on.
static __device__ __align__(256) unsigned char scratch[CONFSPEC_STATIC_SCRATCH_BYTES];

// Settings of one context (confspec_tune).  A new context starts from the defaults below.
struct Settings {
    // Number of leading layers whose GEMM activations carry more than 8 mantissa bits (fp16 operands, or two bf16
    // terms); -1 = derive from the model: the first half of the layers.  The logit error falls steadily with that
    // number (28 layers, d_model 1536, 32 traces: max 0.0176 with 4 such layers, 0.0108 with 8, 0.0062 with 14,
    // 0.0040 with 28) while the pass time rises by 0.6 % from 4 to 14.
    int split_layers = -1;
    // Number of leading layers whose attention runs the two-term variant (q, suffix k / v, probabilities).
    int attn_precise_layers = 1;
    // 1: the last layer's attention rows, output projection and MLP run on the last position of each trace only
    int prune_last_layer = 1;
    // 1: the first layers (the split_layers rule) run their GEMMs on fp16 operands when the packed weights carry
    // fp16 copies; 0: they use two-term bf16 activations against the bf16 weights
    int first_layers_f16 = 1;
    // 1: bf16 models run the QKV projection with the rotary embedding in its epilogue (reordered weight rows)
    int fuse_rope = 1;
    // The gate/up projection warms the last-level cache with the down projection's weights.
    int prefetch_down = 1;
    // A bf16 pass with one new token per trace and at most 32 traces (a generation step) can run on the kernels shaped
    // for it (decode_bf16.hip).  1: it does when d_model and the q width fit one k slice of those kernels (1536), where
    // they win (28 layers x 1536: 1.99 against 2.68 ms per step); wider models stay on the verification pass's kernels,
    // which stream their long k ranges better (64 layers x 5120: 18.7 against 21.6 ms).  2: whenever the shapes allow.
    // 0: never.
    int decode_kernels = 1;
    cs::GemmTune gemm;
    cs::AttnTune attn;
};

static Settings g_default_settings;   // what a new context starts from; changed by confspec_tune(NULL, ...)

// Phase timing (confspec_phase_timing): HIP events recorded on the pass's stream wherever the pass moves from one
// phase to the next; interval i runs from event i to event i + 1 and belongs to phase[i].
struct PhaseTimer {
    bool enabled = false;
    std::vector<hipEvent_t> events;
    std::vector<int> phase;
    int used = 0;          // events recorded by the last pass
    bool overflow = false;
    hipError_t mark(int p, hipStream_t s) {
        if (!enabled) return hipSuccess;
        if (used > 0 && phase[used - 1] == p) return hipSuccess;   // still the same phase
        if (used >= (int)events.size()) { overflow = true; return hipSuccess; }
        phase[used] = p;
        return hipEventRecord(events[used++], s);
    }
};

struct confspec_ctx {
    confspec_model_cfg cfg;
    int device;
    Settings set;
    PhaseTimer timer;
    std::string err;
};

static int split_layers_for(const confspec_ctx *ctx) {
    if (ctx->set.split_layers >= 0) return ctx->set.split_layers;
    return (ctx->cfg.n_layers + 1) / 2;
}

namespace {

int fail(const confspec_ctx *ctx, int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) const_cast<confspec_ctx *>(ctx)->err = buf;
    return code;
}

size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

size_t elem_bytes(int dtype) { return dtype == CONFSPEC_DTYPE_FP32 ? 4 : 2; }

// Workspace layout for a batch of at most T tokens and B traces.
struct WsLayout {
    size_t tok_trace, tok_pos, last_row, rope_cos, rope_sin, x, h, qkv, q, ksuf, vsuf, q_lo, ksuf_lo, vsuf_lo, attn, act;
    size_t plan_counts, plan_tiles, plan_items, part_o, part_ml;
    size_t x_last, h_last, attn_last, act_last, plan2_counts, plan2_tiles, plan2_items;   // last layer, last rows only
    size_t splitk, splitk_bytes;                                                        // split-K partial products
    size_t dec_ctl, dec_ssq;                            // generation-step kernels: control block, partial sums of squares
    size_t part_o_bytes, part_ml_bytes;
    size_t total;
    int64_t max_tiles, max_items, max_tiles2, max_items2;
    size_t slice_off[48], slice_len[48];   // every slice as it was carved, for checks of the layout
    int n_slices;
};

// A pass that the generation-step kernels can take, as far as the model and the batch shape decide it: a bf16 model
// with 128-wide heads, one new token in each of at most 32 traces.
bool dec_shape_ok(const confspec_model_cfg &c, int64_t T, int64_t B) {
    if (c.dtype != CONFSPEC_DTYPE_BF16 || T != B || B < 1 || B > cs::DEC_MAX_ROWS) return false;
    if (c.head_dim != 128 || c.n_kv_heads < 1 || c.n_q_heads % c.n_kv_heads != 0) return false;
    const int G = c.n_q_heads / c.n_kv_heads;
    if (G > cs::DEC_MAX_G || B * c.n_kv_heads > cs::DEC_CTL_TILE - cs::DEC_CTL_ATTN) return false;
    return c.d_model % 64 == 0 && c.d_ffn % 64 == 0 && c.n_layers > 0;
}
// Partial planes of the step's four projections (the largest one).
size_t dec_plane_bytes(const confspec_model_cfg &c) {
    const int qw = c.n_q_heads * c.head_dim, kw = c.n_kv_heads * c.head_dim;
    size_t m = cs::dec_gemm_plane_bytes(c.d_model, (qw + 2 * kw) / 16);
    m = std::max(m, cs::dec_gemm_plane_bytes(qw, c.d_model / 16));
    m = std::max(m, cs::dec_gemm_plane_bytes(c.d_model, c.d_ffn / 8));
    m = std::max(m, cs::dec_gemm_plane_bytes(c.d_ffn, c.d_model / 16));
    return m;
}
// Partial-result records of the step's attention: traces x pieces of the longest trace.
int64_t dec_pieces(const int32_t *h_prefix_lens, int B) {
    int max_L = 0;
    for (int b = 0; b < B; ++b) max_L = std::max(max_L, h_prefix_lens[b]);
    return (int64_t)B * (max_L / cs::DEC_PIECE + 1);
}

// exact (may be null): lay the workspace out for this batch alone instead of for every batch of up to T tokens in B
// traces - the attention plans' lists and partial results and the split-K planes are then sized by what this batch's
// plans and row counts need, which is a small fraction of the general bound (the general bound holds 64 KiB of
// partial results for each of 3 * tiles + 2048 possible pieces).
WsLayout ws_layout(const confspec_ctx *ctx, int64_t T, int64_t B, const confspec_batch *exact = nullptr) {
    const confspec_model_cfg &c = ctx->cfg;
    WsLayout w = {};
    size_t at = 0;
    auto take = [&](size_t bytes) {
        size_t o = at;
        at = align_up(at + bytes);
        if (w.n_slices < 48) { w.slice_off[w.n_slices] = o; w.slice_len[w.n_slices] = bytes; ++w.n_slices; }
        return o;
    };
    size_t eb = elem_bytes(c.dtype);
    size_t qw = (size_t)c.n_q_heads * c.head_dim, kw = (size_t)c.n_kv_heads * c.head_dim;
    w.tok_trace = take(T * 4);
    w.tok_pos = take(T * 4);
    w.last_row = take(B * 4);
    w.rope_cos = take((size_t)T * (c.head_dim / 2) * 4);
    w.rope_sin = take((size_t)T * (c.head_dim / 2) * 4);
    w.x = take((size_t)T * c.d_model * 4);
    size_t terms = c.dtype == CONFSPEC_DTYPE_BF16 ? 2 : 1;   // room for hi | lo activations
    w.h = take((size_t)T * c.d_model * eb * terms);
    w.qkv = take((size_t)T * (qw + 2 * kw) * 4);
    w.q = take((size_t)T * qw * eb);
    w.ksuf = take((size_t)T * kw * eb);
    w.vsuf = take((size_t)T * kw * eb);
    if (c.dtype == CONFSPEC_DTYPE_BF16) {   // second terms for the two-term attention variant
        w.q_lo = take((size_t)T * qw * eb);
        w.ksuf_lo = take((size_t)T * kw * eb);
        w.vsuf_lo = take((size_t)T * kw * eb);
    }
    w.attn = take((size_t)T * qw * eb * terms);
    w.act = take((size_t)T * c.d_ffn * eb * terms);
    if (c.dtype == CONFSPEC_DTYPE_BF16) {
        const int G = c.n_q_heads / c.n_kv_heads;
        cs::attn_plan_capacity(ctx->set.attn, T, B, G, c.n_kv_heads, &w.max_tiles, &w.max_items);
        int64_t part_slots = w.max_items;
        cs::AttnPlanCounts pe = {}, pe_last = {};
        if (exact) {
            pe = cs::attn_plan_counts(ctx->set.attn, exact->h_cu_suffix, exact->h_prefix_lens, exact->B, exact->T, nullptr, 0, G,
                                      c.n_kv_heads, 0);
            pe_last = cs::attn_plan_counts(ctx->set.attn, exact->h_cu_suffix, exact->h_prefix_lens, exact->B, exact->T, nullptr,
                                           0, G, c.n_kv_heads, 1);
            w.max_tiles = std::max<int64_t>(pe.n_tiles, 1);
            w.max_items = std::max<int64_t>(pe.n_items, 1);
            part_slots = std::max<int64_t>(std::max(pe.n_part_slots, pe_last.n_part_slots), 1);
        }
        w.plan_counts = take(256);
        w.plan_tiles = take((size_t)w.max_tiles * sizeof(cs::AttnTile));
        w.plan_items = take((size_t)w.max_items * sizeof(cs::AttnItem));
        w.part_o_bytes = (size_t)part_slots * cs::ATTN_BM * c.head_dim * 4;
        w.part_ml_bytes = (size_t)part_slots * cs::ATTN_BM * 2 * 4;
        if (exact && dec_shape_ok(c, T, B)) {   // the generation-step attention keeps its pieces' partial results here
            int64_t np = dec_pieces(exact->h_prefix_lens, exact->B);
            w.part_o_bytes = std::max(w.part_o_bytes, cs::dec_attn_part_o_bytes(np, c.n_kv_heads));
            w.part_ml_bytes = std::max(w.part_ml_bytes, cs::dec_attn_part_ml_bytes(np, c.n_kv_heads));
        }
        w.part_o = take(w.part_o_bytes);
        w.part_ml = take(w.part_ml_bytes);
        // the last layer works on the last position of each trace only: B rows, one attention tile per
        // trace and kv head (its items fit the partial buffers above: max_items2 <= max_items)
        w.x_last = take((size_t)B * c.d_model * 4);
        w.h_last = take((size_t)B * c.d_model * eb * terms);
        w.attn_last = take((size_t)B * qw * eb * terms);
        w.act_last = take((size_t)B * c.d_ffn * eb * terms);
        w.max_tiles2 = (int64_t)B * c.n_kv_heads;
        w.max_items2 = std::min<int64_t>(w.max_items, 3 * w.max_tiles2 + (w.max_items - 3 * w.max_tiles));
        if (exact) {
            w.max_tiles2 = std::max<int64_t>(pe_last.n_tiles, 1);
            w.max_items2 = std::max<int64_t>(pe_last.n_items, 1);
        }
        w.plan2_counts = take(256);
        w.plan2_tiles = take((size_t)w.max_tiles2 * sizeof(cs::AttnTile));
        w.plan2_items = take((size_t)w.max_items2 * sizeof(cs::AttnItem));
        // partial products of the split-K GEMMs that short row counts take (the B rows of the last layer, a whole
        // pass over few tokens), in both activation widths
        size_t sk = 0;
        for (int t = 1; t <= 2; ++t) {
            if (exact) {   // the projections of this batch run on T rows, or on B rows (last layer)
                for (int rows : {(int)T, (int)B}) {
                    sk = std::max(sk, cs::gemm_splitk_bytes(ctx->set.gemm, rows, (int)(qw + 2 * kw), c.d_model * t));
                    sk = std::max(sk, cs::gemm_splitk_bytes(ctx->set.gemm, rows, c.d_model, (int)qw * t));
                    sk = std::max(sk, cs::gemm_splitk_bytes(ctx->set.gemm, rows, 2 * c.d_ffn, c.d_model * t));
                    sk = std::max(sk, cs::gemm_splitk_bytes(ctx->set.gemm, rows, c.d_model, c.d_ffn * t));
                }
                continue;
            }
            sk = std::max(sk, cs::gemm_splitk_max_bytes(ctx->set.gemm, (int)T, (int)(qw + 2 * kw), c.d_model * t));
            sk = std::max(sk, cs::gemm_splitk_max_bytes(ctx->set.gemm, (int)T, c.d_model, (int)qw * t));
            sk = std::max(sk, cs::gemm_splitk_max_bytes(ctx->set.gemm, (int)T, 2 * c.d_ffn, c.d_model * t));
            sk = std::max(sk, cs::gemm_splitk_max_bytes(ctx->set.gemm, (int)T, c.d_model, c.d_ffn * t));
        }
        // a general layout serves every smaller batch, generation steps included
        if (exact ? dec_shape_ok(c, T, B) : dec_shape_ok(c, 1, 1)) sk = std::max(sk, dec_plane_bytes(c));
        w.splitk_bytes = sk;
        w.splitk = take(std::max<size_t>(sk, 256));
        w.dec_ctl = take((size_t)cs::DEC_CTL_INTS * 4);
        w.dec_ssq = take((size_t)(c.d_model / 16 + 1) * cs::DEC_MAX_ROWS * 4);
    }
    w.total = at;
    return w;
}

// Scratch of the full-vocabulary head for B rows: the last rows of the residual stream, their normalised form (two
// bf16 terms for a bf16 model), the logits [B, vocab], and the verdict outputs the full-vocabulary confidence needs.
struct HeadLayout {
    size_t x, y, logits, v_logits, v_conf, v_verdict, v_accept, part, total;
};
HeadLayout head_layout(const confspec_model_cfg &c, int64_t B) {
    HeadLayout h;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at = align_up(at + bytes); return o; };
    h.x = take((size_t)B * c.d_model * 4);
    h.y = take((size_t)B * c.d_model * 4);           // fp32 rows, or hi | lo bf16 rows: the same size
    h.logits = take((size_t)B * c.vocab * 4);
    h.v_logits = take((size_t)B * CONFSPEC_MAX_VERDICT * 4);
    h.v_conf = take((size_t)B * 4);
    h.v_verdict = take((size_t)B * 4);
    h.v_accept = take((size_t)B);
    h.part = take((size_t)256 * cs::DEC_MAX_ROWS * 4 * 4);   // per-workgroup row statistics of the generation-step head
    h.total = at;
    return h;
}
// What a call wants beyond the verdict outputs.
struct PassExtras {
    const int32_t *dev_n_append = nullptr, *h_n_append = nullptr;   // write-back of suffix keys / values
    const confspec_head_out *head = nullptr;                        // full-vocabulary head at the last positions
    void *head_scratch = nullptr;
    size_t head_scratch_bytes = 0;
    // context units: runs of consecutive traces on one shared context (null: every trace on its own)
    const int32_t *dev_group_start = nullptr, *h_group_start = nullptr;
    int n_groups = 0;
    bool exact_layout = false;                                      // workspace laid out for this batch alone
};

int check_batch(const confspec_ctx *ctx, const confspec_batch *b, int64_t max_prefix, int *max_L_out) {
    if (!b) return fail(ctx, CONFSPEC_E_INVALID_ARG, "batch is null");
    if (b->B < 1 || b->B > (1 << 16)) return fail(ctx, CONFSPEC_E_INVALID_ARG, "B = %d outside [1, 65536]", b->B);
    if (b->T < 1 || b->T > (1 << 22)) return fail(ctx, CONFSPEC_E_INVALID_ARG, "T = %d outside [1, 2^22]", b->T);
    if (!b->suffix_ids || !b->cu_suffix || !b->prefix_lens || !b->h_cu_suffix || !b->h_prefix_lens)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "batch has a null array pointer");
    if (b->h_cu_suffix[0] != 0) return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "cu_suffix[0] = %d, expected 0", b->h_cu_suffix[0]);
    int max_L = 0;
    for (int i = 0; i < b->B; ++i) {
        if (b->h_cu_suffix[i + 1] <= b->h_cu_suffix[i])
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "cu_suffix not strictly increasing at trace %d (every trace needs >= 1 suffix token)", i);
        int L = b->h_prefix_lens[i];
        if (L < 0 || (int64_t)L > max_prefix)
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "prefix_lens[%d] = %d outside [0, %lld] (block table capacity)", i, L, (long long)max_prefix);
        if (L > max_L) max_L = L;
    }
    if (b->h_cu_suffix[b->B] != b->T)
        return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "cu_suffix[B] = %d but T = %d", b->h_cu_suffix[b->B], b->T);
    if (max_L_out) *max_L_out = max_L;
    return CONFSPEC_OK;
}

int check_kv(const confspec_ctx *ctx, const confspec_kv *kv, bool any_prefix) {
    if (!kv) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv is null");
    if (kv->block_size < 1 || kv->max_blocks_per_seq < 1 || kv->n_blocks < 1)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv: block_size, max_blocks_per_seq and n_blocks must be >= 1");
    if (ctx->cfg.dtype == CONFSPEC_DTYPE_BF16 && kv->block_size != 16)
        return fail(ctx, CONFSPEC_E_UNSUPPORTED, "bf16 attention supports block_size 16 only (got %d)", kv->block_size);
    if (!kv->block_table) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv.block_table is null");
    if (any_prefix && (!kv->k_pages || !kv->v_pages)) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv pages are null");
    return CONFSPEC_OK;
}

int check_verdict(const confspec_ctx *ctx, const int32_t *ids, int n, const float *tau, int n_tau,
                  cs::VerdictArgs *va) {
    if (!ids || !tau) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids or tau pointer is null");
    if (n < 2 || n > CONFSPEC_MAX_VERDICT)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "n_verdict = %d outside [2, %d]", n, CONFSPEC_MAX_VERDICT);
    if (n_tau < 1 || n_tau > CONFSPEC_MAX_TAU)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "n_tau = %d outside [1, %d]", n_tau, CONFSPEC_MAX_TAU);
    memset(va, 0, sizeof *va);
    for (int i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= ctx->cfg.vocab)
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "verdict id %d = %d outside [0, %d)", i, ids[i], ctx->cfg.vocab);
        for (int j = 0; j < i; ++j)
            if (ids[j] == ids[i]) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids %d and %d are equal", j, i);
        va->ids[i] = ids[i];
    }
    for (int i = 0; i < n_tau; ++i) {
        if (!(tau[i] >= 0.0f && tau[i] <= 1.0f))
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "tau[%d] = %g outside [0, 1]", i, (double)tau[i]);
        va->tau[i] = tau[i];
    }
    va->n_verdict = n;
    va->n_tau = n_tau;
    return CONFSPEC_OK;
}

int check_ws(const confspec_ctx *ctx, const void *ws, size_t have, size_t need) {
    if (!ws) return fail(ctx, CONFSPEC_E_INVALID_ARG, "workspace is null");
    if (((uintptr_t)ws & 255) != 0) return fail(ctx, CONFSPEC_E_WORKSPACE, "workspace is not 256-byte aligned");
    if (have < need)
        return fail(ctx, CONFSPEC_E_WORKSPACE, "workspace has %zu bytes, %zu needed", have, need);
    return CONFSPEC_OK;
}

// The calling thread's current HIP device must be the one the context was created for: the library never switches
// devices, and kernels launched on another device would read pointers that are not valid there.
int check_device(const confspec_ctx *ctx) {
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e != hipSuccess) return fail(ctx, CONFSPEC_E_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (cur != ctx->device)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "the context was created for device %d but the current device is %d",
                    ctx->device, cur);
    return CONFSPEC_OK;
}

#define HIP_TRY(expr)                                                                                   \
    do {                                                                                                \
        hipError_t e__ = (expr);                                                                        \
        if (e__ != hipSuccess) return fail(ctx, CONFSPEC_E_HIP, "%s: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

int run_gemm(confspec_ctx *ctx, const void *A, const void *W, void *out, int M, int N, int K, int epi,
             int a_terms, int out_terms, hipStream_t s, float *splitk_ws = nullptr, size_t splitk_bytes = 0,
             const cs::PrefetchArgs *pf = nullptr, const cs::NormAfter *norm = nullptr, bool *norm_done = nullptr) {
    if (norm_done) *norm_done = false;
    if (ctx->cfg.dtype == CONFSPEC_DTYPE_FP32) {
        HIP_TRY(cs::launch_gemm_f32((const float *)A, (const float *)W, out, M, N, K, epi, s));
    } else {
        HIP_TRY(cs::launch_gemm_bf16(ctx->set.gemm, (const cs::bf16 *)A, (const cs::bf16 *)W, out, M, N, K, epi, a_terms, out_terms,
                                     splitk_ws, splitk_bytes, s, pf, norm, norm_done));
    }
    return CONFSPEC_OK;
}

cs::AttnArgs make_attn_args(const confspec_model_cfg &c, const confspec_kv *kv, const confspec_batch *b, const int32_t *tok_trace,
                            int layer,
                            const void *q, const void *ksuf, const void *vsuf, const void *q_lo, const void *ksuf_lo,
                            const void *vsuf_lo, void *out, int out_terms) {
    cs::AttnArgs a = {};
    size_t layer_elems = (size_t)kv->n_blocks * c.n_kv_heads * kv->block_size * c.head_dim;
    size_t off = layer_elems * layer * elem_bytes(c.dtype);
    a.q = q; a.ksuf = ksuf; a.vsuf = vsuf; a.out = out;
    a.q_lo = q_lo; a.ksuf_lo = ksuf_lo; a.vsuf_lo = vsuf_lo;
    a.k_pages = kv->k_pages ? (const char *)kv->k_pages + off : nullptr;
    a.v_pages = kv->v_pages ? (const char *)kv->v_pages + off : nullptr;
    a.block_table = kv->block_table;
    a.cu = b->cu_suffix;
    a.plens = b->prefix_lens;
    a.tok_trace = tok_trace;
    a.B = b->B; a.T = b->T; a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads; a.hd = c.head_dim;
    a.n_blocks = kv->n_blocks; a.block_size = kv->block_size; a.max_blocks = kv->max_blocks_per_seq;
    a.scale = 1.0f / sqrtf((float)c.head_dim);
    a.out_terms = out_terms;
    return a;
}

// Attention of one layer on an already planned batch; last_only selects the plan of the last positions.
int run_attention(confspec_ctx *ctx, const cs::AttnArgs &a, char *ws, const WsLayout &L,
                  const cs::AttnPlanCounts &pc, bool last_only, hipStream_t s) {
    if (ctx->cfg.dtype == CONFSPEC_DTYPE_FP32) {
        HIP_TRY(cs::launch_attn_f32(a, (const int32_t *)(ws + L.tok_trace), (const int32_t *)(ws + L.tok_pos), s));
    } else {
        size_t items = last_only ? L.plan2_items : L.plan_items, tiles = last_only ? L.plan2_tiles : L.plan_tiles;
        size_t counts = last_only ? L.plan2_counts : L.plan_counts;
        HIP_TRY(cs::launch_attn_bf16(ctx->set.attn, a, (const cs::AttnItem *)(ws + items), (const int32_t *)(ws + counts),
                                     (int)pc.n_items, (int)pc.max_xcd_items,
                                     (int)(pc.total_chunks / std::max<int64_t>(pc.n_items, 1)), (float *)(ws + L.part_o),
                                     (float *)(ws + L.part_ml), s));
        if (pc.n_part_slots > 0) {
            HIP_TRY(ctx->timer.mark(CONFSPEC_PHASE_ATTN_MERGE, s));
            HIP_TRY(cs::launch_attn_merge(a, (const cs::AttnTile *)(ws + tiles), (const int32_t *)(ws + counts),
                                          (int)pc.n_tiles, (const float *)(ws + L.part_o), (const float *)(ws + L.part_ml), s));
        }
    }
    return CONFSPEC_OK;
}

// One attention plan (bf16 only): all suffix rows, or the last position of each trace.
struct Groups {
    const int32_t *dev = nullptr, *host = nullptr;
    int n = 0;
};
int run_attn_plan(confspec_ctx *ctx, const confspec_batch *b, const Groups &gr, int max_L, char *ws, const WsLayout &L,
                  bool last_only, cs::AttnPlanCounts *pc, hipStream_t s) {
    const confspec_model_cfg &c = ctx->cfg;
    int G = c.n_q_heads / c.n_kv_heads;
    int64_t cap_tiles = last_only ? L.max_tiles2 : L.max_tiles, cap_items = last_only ? L.max_items2 : L.max_items;
    *pc = cs::attn_plan_counts(ctx->set.attn, b->h_cu_suffix, b->h_prefix_lens, b->B, b->T, gr.host, gr.n, G, c.n_kv_heads,
                               last_only ? 1 : 0);
    if (pc->n_tiles > cap_tiles || pc->n_items > cap_items)
        return fail(ctx, CONFSPEC_E_WORKSPACE, "attention plan (%lld tiles, %lld items) exceeds workspace capacity",
                    (long long)pc->n_tiles, (long long)pc->n_items);
    HIP_TRY(cs::launch_attn_plan(b->cu_suffix, b->prefix_lens, gr.dev, gr.n, b->B, b->T, max_L, G, c.n_kv_heads, pc->chunks_per_item,
                                 pc->equalize, last_only ? 1 : 0, (int)cap_tiles, (int)cap_items,
                                 (cs::AttnTile *)(ws + (last_only ? L.plan2_tiles : L.plan_tiles)),
                                 (cs::AttnItem *)(ws + (last_only ? L.plan2_items : L.plan_items)),
                                 (int32_t *)(ws + (last_only ? L.plan2_counts : L.plan_counts)), s));
    return CONFSPEC_OK;
}

// prep + (bf16) attention plan of all rows; fills pc.
int run_plan(confspec_ctx *ctx, const confspec_batch *b, const Groups &gr, int max_L, char *ws, const WsLayout &L,
             cs::AttnPlanCounts *pc, hipStream_t s) {
    const confspec_model_cfg &c = ctx->cfg;
    HIP_TRY(cs::launch_prep(b->cu_suffix, b->prefix_lens, b->B, b->T, max_L, (int32_t *)(ws + L.tok_trace),
                            (int32_t *)(ws + L.tok_pos), (int32_t *)(ws + L.last_row), s));
    *pc = cs::AttnPlanCounts{};
    if (c.dtype == CONFSPEC_DTYPE_BF16) return run_attn_plan(ctx, b, gr, max_L, ws, L, false, pc, s);
    return CONFSPEC_OK;
}

}  // namespace

extern "C" {

const char *confspec_version(void) { return "0.1"; }

int confspec_create(const confspec_model_cfg *cfg, int device, confspec_ctx **out) {
    if (!cfg || !out) return CONFSPEC_E_INVALID_ARG;
    *out = nullptr;
    const confspec_model_cfg &c = *cfg;
    if (c.n_layers < 0 || c.d_model < 1 || c.n_q_heads < 1 || c.n_kv_heads < 1 || c.head_dim < 1 || c.d_ffn < 1 ||
        c.vocab < 1 || !(c.rope_theta > 0.f) || !(c.rms_eps >= 0.f) || device < 0)
        return CONFSPEC_E_INVALID_ARG;
    if (c.dtype != CONFSPEC_DTYPE_FP32 && c.dtype != CONFSPEC_DTYPE_BF16) return CONFSPEC_E_UNSUPPORTED;
    if (c.n_q_heads % c.n_kv_heads != 0) return CONFSPEC_E_UNSUPPORTED;
    int qkv = (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, qw = c.n_q_heads * c.head_dim;
    if (c.dtype == CONFSPEC_DTYPE_BF16) {
        if (c.head_dim != 128) return CONFSPEC_E_UNSUPPORTED;
        if (c.d_model % 128 || c.d_ffn % 64 || qkv % 128 || qw % 64) return CONFSPEC_E_UNSUPPORTED;
    } else {
        if (c.head_dim != 64 && c.head_dim != 128) return CONFSPEC_E_UNSUPPORTED;
        if (c.d_model % 64 || c.d_ffn % 32 || qkv % 64 || qw % 16) return CONFSPEC_E_UNSUPPORTED;
    }
    confspec_ctx *ctx = new (std::nothrow) confspec_ctx();
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    ctx->cfg = c;
    ctx->device = device;
    ctx->set = g_default_settings;
    *out = ctx;
    return CONFSPEC_OK;
}

void confspec_destroy(confspec_ctx *ctx) {
    if (!ctx) return;
    for (hipEvent_t e : ctx->timer.events) (void)hipEventDestroy(e);
    delete ctx;
}

const char *confspec_last_error(const confspec_ctx *ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int confspec_workspace_bytes(const confspec_ctx *ctx, int32_t max_T, int32_t max_B, int64_t max_sum_L,
                             size_t *out_bytes) {
    if (!ctx || !out_bytes) return CONFSPEC_E_INVALID_ARG;
    if (max_T < 1 || max_B < 1 || max_sum_L < 0) return fail(ctx, CONFSPEC_E_INVALID_ARG, "max_T, max_B must be >= 1, max_sum_L >= 0");
    *out_bytes = ws_layout(ctx, max_T, max_B).total;
    return CONFSPEC_OK;
}

namespace {
// fp16 copies are made for the layers that would otherwise run with two-term activations
int f16_layers_for(const confspec_ctx *ctx) {
    const confspec_model_cfg &c = ctx->cfg;
    if (c.dtype != CONFSPEC_DTYPE_BF16 || !ctx->set.first_layers_f16) return 0;
    return std::min(c.n_layers, split_layers_for(ctx));
}
struct PackLayout {
    size_t gate_up;        // bytes of one packed gate/up matrix (aligned)
    size_t qkv_perm;       // bytes of one reordered wqkv matrix (aligned; bf16 models only, else 0)
    size_t f16[4];         // bytes of the fp16 copies of wqkv, wo, gate/up, down (aligned)
    size_t elems[4];
    size_t total;
};
PackLayout pack_layout(const confspec_ctx *ctx) {
    const confspec_model_cfg &c = ctx->cfg;
    PackLayout p = {};
    size_t qw = (size_t)c.n_q_heads * c.head_dim, kw = (size_t)c.n_kv_heads * c.head_dim;
    p.gate_up = align_up((size_t)2 * c.d_ffn * c.d_model * elem_bytes(c.dtype));
    p.elems[0] = (qw + 2 * kw) * c.d_model;
    p.elems[1] = (size_t)c.d_model * qw;
    p.elems[2] = (size_t)2 * c.d_ffn * c.d_model;
    p.elems[3] = (size_t)c.d_model * c.d_ffn;
    size_t per16 = 0;
    for (int i = 0; i < 4; ++i) { p.f16[i] = align_up(p.elems[i] * 2); per16 += p.f16[i]; }
    p.qkv_perm = c.dtype == CONFSPEC_DTYPE_BF16 ? align_up(p.elems[0] * 2) : 0;
    p.total = (size_t)c.n_layers * (p.gate_up + p.qkv_perm) + (size_t)f16_layers_for(ctx) * per16;
    return p;
}
}  // namespace

int confspec_packed_bytes(const confspec_ctx *ctx, size_t *out_bytes) {
    if (!ctx || !out_bytes) return CONFSPEC_E_INVALID_ARG;
    *out_bytes = pack_layout(ctx).total;
    return CONFSPEC_OK;
}

int confspec_pack_weights(confspec_ctx *ctx, const confspec_weights *in, void *dev_dst, size_t dst_bytes,
                          const void **h_ptr_storage, confspec_weights *out, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!in || !out || !h_ptr_storage) return fail(ctx, CONFSPEC_E_INVALID_ARG, "null argument");
    if (in->packed != 0) return fail(ctx, CONFSPEC_E_INVALID_ARG, "input weights are already packed");
    const confspec_model_cfg &c = ctx->cfg;
    if (c.d_ffn % 32) return fail(ctx, CONFSPEC_E_UNSUPPORTED, "d_ffn must be a multiple of 32");
    PackLayout P = pack_layout(ctx);
    if (!dev_dst || ((uintptr_t)dev_dst & 255)) return fail(ctx, CONFSPEC_E_WORKSPACE, "dev_dst null or not 256-byte aligned");
    if (dst_bytes < P.total) return fail(ctx, CONFSPEC_E_WORKSPACE, "dev_dst has %zu bytes, %zu needed", dst_bytes, P.total);
    if (c.n_layers > 0 && !in->w_gate_up) return fail(ctx, CONFSPEC_E_INVALID_ARG, "w_gate_up is null");
    int n16 = f16_layers_for(ctx);
    const bool bf = c.dtype == CONFSPEC_DTYPE_BF16;
    if (c.n_layers > 0 && ((bf && !in->wqkv) || (n16 > 0 && (!in->wo || !in->w_down))))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "a per-layer weight array is null");
    for (int l = 0; l < c.n_layers; ++l) {
        if (!in->w_gate_up[l]) return fail(ctx, CONFSPEC_E_INVALID_ARG, "w_gate_up[%d] is null", l);
        if ((bf && !in->wqkv[l]) || (l < n16 && (!in->wo[l] || !in->w_down[l])))
            return fail(ctx, CONFSPEC_E_INVALID_ARG, "layer %d has a null weight pointer", l);
    }
    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    const int n = c.n_layers;
    for (int i = 0; i < 6 * n; ++i) h_ptr_storage[i] = nullptr;
    char *at = (char *)dev_dst;
    for (int l = 0; l < n; ++l) {
        HIP_TRY(cs::launch_pack_gate_up(c.dtype, in->w_gate_up[l], at, c.d_ffn, c.d_model, s));
        h_ptr_storage[l] = at;
        at += P.gate_up;
    }
    if (bf)
        for (int l = 0; l < n; ++l) {
            HIP_TRY(cs::launch_permute_heads(in->wqkv[l], at, c.n_q_heads + 2 * c.n_kv_heads, c.d_model, s));
            h_ptr_storage[5 * n + l] = at;
            at += P.qkv_perm;
        }
    for (int l = 0; l < n16; ++l) {
        const void *src[4] = {h_ptr_storage[5 * n + l] /* reordered */, in->wo[l], h_ptr_storage[l] /* packed order */,
                              in->w_down[l]};
        for (int i = 0; i < 4; ++i) {
            HIP_TRY(cs::launch_bf16_to_f16(src[i], at, P.elems[i], s));
            h_ptr_storage[(1 + i) * n + l] = at;
            at += P.f16[i];
        }
    }
    *out = *in;
    out->w_gate_up = h_ptr_storage;
    out->packed = 1;
    out->n_f16_layers = n16;
    out->wqkv_f16 = h_ptr_storage + n;
    out->wo_f16 = h_ptr_storage + 2 * n;
    out->w_gate_up_f16 = h_ptr_storage + 3 * n;
    out->w_down_f16 = h_ptr_storage + 4 * n;
    out->wqkv_perm = bf ? h_ptr_storage + 5 * n : nullptr;
    return CONFSPEC_OK;
}

// The pass; with dev_n_append it also writes the keys and values of the first n_append[b] suffix tokens of every
// trace back into the cache (h_n_append: the same counts on the host, for validation).
static int verify_impl(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                       const confspec_batch *batch, const int32_t *h_verdict_ids, int32_t n_verdict,
                       const float *h_tau, int32_t n_tau, void *dev_workspace, size_t workspace_bytes,
                       float *dev_verdict_logits, float *dev_conf, int32_t *dev_verdict, uint8_t *dev_accept,
                       const PassExtras &ex, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    const confspec_model_cfg &c = ctx->cfg;
    const int32_t *dev_n_append = ex.dev_n_append, *h_n_append = ex.h_n_append;
    const bool want_verdict = h_verdict_ids != nullptr;     // a generation step may come without verdict tokens
    if (!w) return fail(ctx, CONFSPEC_E_INVALID_ARG, "weights is null");
    if (!ex.head && (!dev_verdict_logits || !dev_conf || !dev_verdict || !dev_accept))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "an output pointer is null");
    if (w->packed != 1) return fail(ctx, CONFSPEC_E_INVALID_ARG, "weights must be packed with confspec_pack_weights");
    if (!w->embed || !w->lm_head || !w->final_norm) return fail(ctx, CONFSPEC_E_INVALID_ARG, "embed, lm_head or final_norm is null");
    if (c.n_layers > 0 && (!w->attn_norm || !w->wqkv || !w->wo || !w->mlp_norm || !w->w_gate_up || !w->w_down))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "a per-layer weight array is null");
    for (int l = 0; l < c.n_layers; ++l)
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->mlp_norm[l] || !w->w_gate_up[l] || !w->w_down[l])
            return fail(ctx, CONFSPEC_E_INVALID_ARG, "layer %d has a null weight pointer", l);
    int rc;
    if (!kv) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv is null");
    int max_L = 0;
    int64_t max_prefix = (int64_t)kv->max_blocks_per_seq * kv->block_size;
    if ((rc = check_batch(ctx, batch, max_prefix, &max_L)) != CONFSPEC_OK) return rc;
    if ((rc = check_kv(ctx, kv, max_L > 0)) != CONFSPEC_OK) return rc;
    cs::VerdictArgs va = {};
    if (want_verdict && (rc = check_verdict(ctx, h_verdict_ids, n_verdict, h_tau, n_tau, &va)) != CONFSPEC_OK) return rc;
    WsLayout L = ws_layout(ctx, batch->T, batch->B, ex.exact_layout ? batch : nullptr);
    if ((rc = check_ws(ctx, dev_workspace, workspace_bytes, L.total)) != CONFSPEC_OK) return rc;
    HeadLayout HL = {};
    if (ex.head) {
        if (!ex.head->token || !ex.head->max_logit || !ex.head->lse) return fail(ctx, CONFSPEC_E_INVALID_ARG, "a head output pointer is null");
        if (ex.head->conf_full && !want_verdict)
            return fail(ctx, CONFSPEC_E_INVALID_ARG, "conf_full needs verdict ids");
        if (c.dtype == CONFSPEC_DTYPE_BF16 ? (c.vocab % 128 != 0) : (c.vocab % 64 != 0))
            return fail(ctx, CONFSPEC_E_UNSUPPORTED, "the full-vocabulary head needs vocab %% %d == 0 (got %d)",
                        c.dtype == CONFSPEC_DTYPE_BF16 ? 128 : 64, c.vocab);
        HL = head_layout(c, batch->B);
        if ((rc = check_ws(ctx, ex.head_scratch, ex.head_scratch_bytes, HL.total)) != CONFSPEC_OK) return rc;
    }
    if (ex.dev_group_start || ex.h_group_start) {
        if (!ex.dev_group_start || !ex.h_group_start) return fail(ctx, CONFSPEC_E_INVALID_ARG, "group_start needs its dev and host copy");
        const int32_t *gs = ex.h_group_start;
        if (ex.n_groups < 1 || ex.n_groups > batch->B)
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "n_groups = %d outside [1, B = %d]", ex.n_groups, batch->B);
        if (gs[0] != 0 || gs[ex.n_groups] != batch->B)
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "group_start must run from 0 to B = %d (got %d .. %d)", batch->B, gs[0], gs[ex.n_groups]);
        for (int g = 0; g < ex.n_groups; ++g) {
            if (gs[g + 1] <= gs[g]) return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "group_start not strictly increasing at group %d", g);
            for (int b = gs[g] + 1; b < gs[g + 1]; ++b)
                if (batch->h_prefix_lens[b] != batch->h_prefix_lens[gs[g]])
                    return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "traces %d and %d of group %d have different prefix lengths (%d, %d)",
                                gs[g], b, g, batch->h_prefix_lens[gs[g]], batch->h_prefix_lens[b]);
        }
        if (c.dtype != CONFSPEC_DTYPE_BF16) return fail(ctx, CONFSPEC_E_UNSUPPORTED, "shared-context groups need a bf16 context");
    }
    if (dev_n_append) {
        if (!h_n_append) return fail(ctx, CONFSPEC_E_INVALID_ARG, "h_n_append is null");
        if (!kv->k_pages || !kv->v_pages) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv pages are null");
        for (int b = 0; b < batch->B; ++b) {
            int n = h_n_append[b], S = batch->h_cu_suffix[b + 1] - batch->h_cu_suffix[b];
            if (n < 0 || n > S) return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "n_append[%d] = %d outside [0, S_b = %d]", b, n, S);
            if ((int64_t)batch->h_prefix_lens[b] + n > max_prefix)
                return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "trace %d: %d cached + %d appended rows exceed the block table's %lld",
                            b, batch->h_prefix_lens[b], n, (long long)max_prefix);
        }
    }

    if ((rc = check_device(ctx)) != CONFSPEC_OK) return rc;
    hipStream_t s = (hipStream_t)stream;
    char *ws = (char *)dev_workspace;
    int T = batch->T, B = batch->B, d = c.d_model;
    int qw = c.n_q_heads * c.head_dim, kw = c.n_kv_heads * c.head_dim;
    float *x = (float *)(ws + L.x);
    void *h = ws + L.h;
    float *qkv = (float *)(ws + L.qkv);

    // phase timing: an event at every change of phase (only when switched on; never under stream capture)
    PhaseTimer &tm_ = ctx->timer;
    tm_.used = 0;
    tm_.overflow = false;
    auto mark = [&](int phase) -> hipError_t { return tm_.mark(phase, s); };
    HIP_TRY(mark(CONFSPEC_PHASE_OTHER));
    const Settings &set = ctx->set;
    size_t eb = elem_bytes(c.dtype);
    // Activation format of a layer's GEMMs (see gemm_bf16.hip): the first layers run on fp16 operands when the
    // packed weights carry fp16 copies (3), else with two bf16 terms (2); the rest is plain bf16 (1).
    // The projection kernel that rotates q and k itself reads wqkv with reordered rows (the half copy has that
    // order too, so fp16 layers depend on it).
    auto rope_fused_in = [&](int l) {
        return c.dtype == CONFSPEC_DTYPE_BF16 && set.fuse_rope && c.head_dim == 128 && w->wqkv_perm && w->wqkv_perm[l];
    };
    auto format_of = [&](int l) {
        if (!(c.dtype == CONFSPEC_DTYPE_BF16 && l < split_layers_for(ctx))) return 1;
        if (rope_fused_in(l) && set.first_layers_f16 && l < w->n_f16_layers && w->wqkv_f16 && w->wo_f16 && w->w_gate_up_f16 &&
            w->w_down_f16 && w->wqkv_f16[l] && w->wo_f16[l] && w->w_gate_up_f16[l] && w->w_down_f16[l])
            return 3;
        return 2;
    };
    // A generation step (one new token per trace, at most 32 traces) runs on the kernels shaped for it when every
    // layer's operands are single 16-bit values (bf16 or fp16) and the scratch holds its partial results; everything
    // else, and any step that does not fit, takes the general kernels below.
    bool use_dec = set.decode_kernels && dec_shape_ok(c, T, B) && !ex.dev_group_start &&
                   (set.decode_kernels == 2 || (d <= 64 * cs::DEC_MAX_KT && qw <= 64 * cs::DEC_MAX_KT));
    int64_t dec_np = 0;
    if (use_dec) {
        for (int l = 0; l < c.n_layers && use_dec; ++l) use_dec = rope_fused_in(l) && format_of(l) != 2;
        dec_np = dec_pieces(batch->h_prefix_lens, B);
        use_dec = use_dec && dec_plane_bytes(c) <= L.splitk_bytes && cs::dec_attn_part_o_bytes(dec_np, c.n_kv_heads) <= L.part_o_bytes &&
                  cs::dec_attn_part_ml_bytes(dec_np, c.n_kv_heads) <= L.part_ml_bytes;
    }
    cs::AttnPlanCounts pc = {}, pc_last = {};
    Groups gr;
    gr.dev = ex.dev_group_start; gr.host = ex.h_group_start; gr.n = ex.n_groups;
    // Only the last position of each trace feeds the verdict head, so everything of the last layer that
    // comes after its keys and values - attention rows, output projection, MLP - runs on those B rows.
    const bool prune = c.dtype == CONFSPEC_DTYPE_BF16 && set.prune_last_layer && c.n_layers > 0;
    if (use_dec) {   // the generation-step attention has its own, fixed cut into pieces: no plan
        HIP_TRY(cs::launch_prep(batch->cu_suffix, batch->prefix_lens, B, T, max_L, (int32_t *)(ws + L.tok_trace),
                                (int32_t *)(ws + L.tok_pos), (int32_t *)(ws + L.last_row), s));
    } else {
        if ((rc = run_plan(ctx, batch, gr, max_L, ws, L, &pc, s)) != CONFSPEC_OK) return rc;
        if (prune && (rc = run_attn_plan(ctx, batch, gr, max_L, ws, L, true, &pc_last, s)) != CONFSPEC_OK) return rc;
    }
    HIP_TRY(cs::launch_rope_table((const int32_t *)(ws + L.tok_pos), T, c.head_dim, c.rope_theta,
                                  (float *)(ws + L.rope_cos), (float *)(ws + L.rope_sin), s));
    HIP_TRY(cs::launch_embed(c.dtype, batch->suffix_ids, w->embed, x, T, d, c.vocab, s));
    const int32_t *last_row = (const int32_t *)(ws + L.last_row);
    if (use_dec) {
        int32_t *ctl = (int32_t *)(ws + L.dec_ctl);
        HIP_TRY(cs::launch_dec_init(ctl, s));
        const size_t layer_bytes = (size_t)kv->n_blocks * c.n_kv_heads * kv->block_size * c.head_dim * eb;
        // The RMSNorm in front of the QKV and gate/up projections: the residual projection before writes x * gain in
        // the operand format and per-row partial sums of squares, the consumer scales its result rows (decode_bf16.hip).
        // The first layer's input comes from the embedding: the RMSNorm kernel, once.
        float *ssq = (float *)(ws + L.dec_ssq);
        const int ssq_n = d / 16;
        HIP_TRY(mark(CONFSPEC_PHASE_NORM));
        HIP_TRY(cs::launch_rmsnorm(c.dtype, x, w->attn_norm[0], h, T, d, c.rms_eps, format_of(0), s));
        auto proj = [&](cs::DecGemm &g, const void *X, int ldx, const void *W, int K, int n_ct) {
            g.X = (const cs::bf16 *)X; g.ldx = ldx; g.W = (const cs::bf16 *)W; g.M = B; g.K = K; g.n_ct = n_ct;
            cs::dec_gemm_plan(K, n_ct, &g.S, &g.nwg);
            g.planes = (float *)(ws + L.splitk);
            g.tile_cnt = ctl + cs::DEC_CTL_TILE;
        };
        for (int l = 0; l < c.n_layers; ++l) {
            const int tm = format_of(l);
            const bool f16 = tm == 3;
            const void *wqkv = f16 ? w->wqkv_f16[l] : w->wqkv_perm[l], *wo = f16 ? w->wo_f16[l] : w->wo[l];
            const void *wgu = f16 ? w->w_gate_up_f16[l] : w->w_gate_up[l], *wdn = f16 ? w->w_down_f16[l] : w->w_down[l];
            HIP_TRY(mark(CONFSPEC_PHASE_QKV));
            cs::DecGemm gq = {};
            proj(gq, h, d, wqkv, d, (qw + 2 * kw) / 16);
            if (l > 0) { gq.ssq_in = ssq; gq.ssq_n = ssq_n; gq.eps = c.rms_eps; }
            gq.rope = cs::RopeArgs{(const float *)(ws + L.rope_cos), (const float *)(ws + L.rope_sin), ws + L.q, ws + L.ksuf, ws + L.vsuf,
                                   ws + L.q_lo, nullptr, nullptr, c.n_q_heads, c.n_kv_heads};
            gq.perm = 1;
            if (dev_n_append) {
                gq.k_pages = (char *)const_cast<void *>(kv->k_pages) + layer_bytes * l;
                gq.v_pages = (char *)const_cast<void *>(kv->v_pages) + layer_bytes * l;
                gq.table = kv->block_table; gq.plens = batch->prefix_lens; gq.n_append = dev_n_append;
                gq.max_blocks = kv->max_blocks_per_seq; gq.n_blocks = kv->n_blocks;
            }
            HIP_TRY(cs::launch_dec_gemm(gq, cs::DEC_EPI_ROPE, f16, s));
            HIP_TRY(mark(CONFSPEC_PHASE_ATTN));
            cs::DecAttn at = {};
            at.q = (const cs::bf16 *)(ws + L.q); at.q_lo = (const cs::bf16 *)(ws + L.q_lo);
            at.ksuf = (const cs::bf16 *)(ws + L.ksuf); at.vsuf = (const cs::bf16 *)(ws + L.vsuf);
            at.k_pages = kv->k_pages ? (const cs::bf16 *)((const char *)kv->k_pages + layer_bytes * l) : nullptr;
            at.v_pages = kv->v_pages ? (const cs::bf16 *)((const char *)kv->v_pages + layer_bytes * l) : nullptr;
            at.table = kv->block_table; at.plens = batch->prefix_lens; at.ctl = ctl;
            at.out = ws + L.attn; at.out_fmt = tm;
            at.part_o = (float *)(ws + L.part_o); at.part_ml = (float *)(ws + L.part_ml);
            at.B = B; at.Hq = c.n_q_heads; at.Hkv = c.n_kv_heads; at.G = c.n_q_heads / c.n_kv_heads;
            at.max_blocks = kv->max_blocks_per_seq; at.n_blocks = kv->n_blocks; at.max_L = max_L;
            at.scale_log2 = 1.44269504088896340736f / sqrtf((float)c.head_dim);
            at.n_iter = cs::dec_attn_rounds(B, c.n_kv_heads, max_L);
            at.max_pieces = max_L / (cs::DEC_PIECE * at.n_iter) + 1;
            HIP_TRY(cs::launch_dec_attn(at, s));
            HIP_TRY(mark(CONFSPEC_PHASE_O_PROJ));
            cs::DecGemm go = {};
            proj(go, ws + L.attn, qw, wo, qw, d / 16);
            go.x = x; go.xg_out = h; go.g_next = (const cs::bf16 *)w->mlp_norm[l]; go.ssq_out = ssq; go.xg_fmt = tm;
            HIP_TRY(cs::launch_dec_gemm(go, cs::DEC_EPI_RESID, f16, s));
            HIP_TRY(mark(CONFSPEC_PHASE_GATE_UP));
            cs::DecGemm gg = {};
            proj(gg, h, d, wgu, d, c.d_ffn / 8);
            gg.ssq_in = ssq; gg.ssq_n = ssq_n; gg.eps = c.rms_eps;
            gg.act = ws + L.act; gg.act_fmt = tm;
            HIP_TRY(cs::launch_dec_gemm(gg, cs::DEC_EPI_SWIGLU, f16, s));
            HIP_TRY(mark(CONFSPEC_PHASE_DOWN));
            cs::DecGemm gd = {};
            proj(gd, ws + L.act, c.d_ffn, wdn, c.d_ffn, d / 16);
            gd.x = x;
            if (l + 1 < c.n_layers) {   // the next layer's operand, in that layer's format
                gd.xg_out = h; gd.g_next = (const cs::bf16 *)w->attn_norm[l + 1]; gd.ssq_out = ssq; gd.xg_fmt = format_of(l + 1);
            }
            HIP_TRY(cs::launch_dec_gemm(gd, cs::DEC_EPI_RESID, f16, s));
        }
    }
    bool attn_norm_done = false;   // the previous layer's down projection already wrote this layer's normalised input
    for (int l = 0; l < c.n_layers && !use_dec; ++l) {
        const int tm = format_of(l);
        const void *wqkv = w->wqkv[l], *wo = w->wo[l], *wgu = w->w_gate_up[l], *wdn = w->w_down[l];
        const bool rope_fused = rope_fused_in(l);
        if (tm == 3) {
            wqkv = w->wqkv_f16[l]; wo = w->wo_f16[l]; wgu = w->w_gate_up_f16[l]; wdn = w->w_down_f16[l];
        }
        const int wide = tm == 2 ? 2 : 1;      // buffer width multiplier of the activation format
        bool prec = c.dtype == CONFSPEC_DTYPE_BF16 && l < set.attn_precise_layers;
        bool last = prune && l == c.n_layers - 1;
        float *sk = c.dtype == CONFSPEC_DTYPE_BF16 ? (float *)(ws + L.splitk) : nullptr;   // for outputs of few tiles
        size_t skb = sk ? L.splitk_bytes : 0;
        HIP_TRY(mark(CONFSPEC_PHASE_NORM));
        if (!attn_norm_done) HIP_TRY(cs::launch_rmsnorm(c.dtype, x, w->attn_norm[l], h, T, d, c.rms_eps, tm, s));
        attn_norm_done = false;
        HIP_TRY(mark(CONFSPEC_PHASE_QKV));
        if (rope_fused) {
            cs::RopeArgs ra = {(const float *)(ws + L.rope_cos), (const float *)(ws + L.rope_sin), ws + L.q, ws + L.ksuf,
                               ws + L.vsuf, prec ? ws + L.q_lo : nullptr, prec ? ws + L.ksuf_lo : nullptr,
                               prec ? ws + L.vsuf_lo : nullptr, c.n_q_heads, c.n_kv_heads};
            HIP_TRY(cs::launch_gemm_bf16_rope(set.gemm, (const cs::bf16 *)h, (const cs::bf16 *)(tm == 3 ? wqkv : w->wqkv_perm[l]), T,
                                              qw + 2 * kw, d, tm, ra, sk, skb, s));
        } else {
            if ((rc = run_gemm(ctx, h, wqkv, qkv, T, qw + 2 * kw, d, cs::EPI_STORE_F32, tm, 1, s, sk, skb))) return rc;
            HIP_TRY(cs::launch_rope_split(c.dtype, qkv, (const float *)(ws + L.rope_cos), (const float *)(ws + L.rope_sin),
                                          ws + L.q, ws + L.ksuf, ws + L.vsuf, prec ? ws + L.q_lo : nullptr,
                                          prec ? ws + L.ksuf_lo : nullptr, prec ? ws + L.vsuf_lo : nullptr, T, c.n_q_heads,
                                          c.n_kv_heads, c.head_dim, s));
        }
        cs::AttnArgs a = make_attn_args(c, kv, batch, (const int32_t *)(ws + L.tok_trace), l, ws + L.q, ws + L.ksuf, ws + L.vsuf, prec ? ws + L.q_lo : nullptr,
                                        prec ? ws + L.ksuf_lo : nullptr, prec ? ws + L.vsuf_lo : nullptr, ws + L.attn, tm);
        HIP_TRY(mark(prec ? CONFSPEC_PHASE_ATTN_PRECISE : CONFSPEC_PHASE_ATTN));
        if ((rc = run_attention(ctx, a, ws, L, last ? pc_last : pc, last, s))) return rc;
        HIP_TRY(mark(CONFSPEC_PHASE_OTHER));
        if (dev_n_append) {
            // after this layer's attention has read the pages (it never reads rows at or past L_b anyway)
            size_t layer_bytes = (size_t)kv->n_blocks * c.n_kv_heads * kv->block_size * c.head_dim * eb;
            HIP_TRY(cs::launch_kv_append(ws + L.ksuf, ws + L.vsuf, (char *)const_cast<void *>(kv->k_pages) + layer_bytes * l,
                                         (char *)const_cast<void *>(kv->v_pages) + layer_bytes * l, kv->block_table,
                                         batch->cu_suffix, batch->prefix_lens, dev_n_append,
                                         (const int32_t *)(ws + L.tok_trace), B, T, c.n_kv_heads, (size_t)c.head_dim * eb,
                                         kv->block_size, kv->max_blocks_per_seq, kv->n_blocks, s));
        }
        float *xr = x;             // residual stream the rest of the layer works on
        const void *attn = ws + L.attn;
        void *hr = h, *act = ws + L.act;
        int rows = T;
        if (last) {
            xr = (float *)(ws + L.x_last); hr = ws + L.h_last; act = ws + L.act_last; rows = B;
            HIP_TRY(cs::launch_gather_rows(x, xr, last_row, B, T, (size_t)d * 4, s));
            HIP_TRY(cs::launch_gather_rows(ws + L.attn, ws + L.attn_last, last_row, B, T, (size_t)qw * eb * wide, s));
            attn = ws + L.attn_last;
        }
        // A residual projection that takes the split-K path (few rows) writes the following RMSNorm along with the
        // residual update; otherwise the RMSNorm is a kernel of its own.
        cs::NormAfter na;
        na.g = w->mlp_norm[l]; na.h = hr; na.eps = c.rms_eps; na.terms = tm;
        bool mlp_norm_done = false;
        HIP_TRY(mark(CONFSPEC_PHASE_O_PROJ));
        if ((rc = run_gemm(ctx, attn, wo, xr, rows, d, qw, cs::EPI_RESID_F32, tm, 1, s, sk, skb, nullptr, &na, &mlp_norm_done))) return rc;
        HIP_TRY(mark(CONFSPEC_PHASE_NORM));
        if (!mlp_norm_done) HIP_TRY(cs::launch_rmsnorm(c.dtype, xr, w->mlp_norm[l], hr, rows, d, c.rms_eps, tm, s));
        // the gate/up projection is compute-bound: while it runs it also pulls the down projection's weights, which
        // that kernel reads in strided pieces, into the last-level cache
        // (a down projection cut into k slices of 256 x 256 tiles reads whole 128-byte lines of 256 rows at a time and
        // does not gain from it: config 2 is 0.5 % faster without the hint, the unsplit shapes 0.1-0.2 % slower)
        bool big_tiles = false;
        const bool warm = set.prefetch_down && !(sk && cs::gemm_splitk_factor(set.gemm, rows, d, c.d_ffn * wide, &big_tiles) > 1);
        cs::PrefetchArgs pf;
        pf.ptr = warm ? wdn : nullptr;
        pf.n16 = warm ? (unsigned)((size_t)d * c.d_ffn * eb / 16) : 0u;
        HIP_TRY(mark(CONFSPEC_PHASE_GATE_UP));
        if ((rc = run_gemm(ctx, hr, wgu, act, rows, 2 * c.d_ffn, d, cs::EPI_SWIGLU, tm, tm, s, sk, skb, &pf))) return rc;
        HIP_TRY(mark(CONFSPEC_PHASE_DOWN));
        cs::NormAfter nb;
        const bool has_next = !last && l + 1 < c.n_layers;        // rows == T: the next layer normalises the same rows
        if (has_next) { nb.g = w->attn_norm[l + 1]; nb.h = h; nb.eps = c.rms_eps; nb.terms = format_of(l + 1); }
        if ((rc = run_gemm(ctx, act, wdn, xr, rows, d, c.d_ffn, cs::EPI_RESID_F32, tm, 1, s, sk, skb, nullptr,
                           has_next ? &nb : nullptr, &attn_norm_done)))
            return rc;
    }
    HIP_TRY(mark(CONFSPEC_PHASE_OTHER));
    if (ex.head) {   // verdict outputs, if any, go to the head's scratch
        char *hs = (char *)ex.head_scratch;
        dev_verdict_logits = (float *)(hs + HL.v_logits);
        dev_conf = (float *)(hs + HL.v_conf);
        dev_verdict = (int32_t *)(hs + HL.v_verdict);
        dev_accept = (uint8_t *)(hs + HL.v_accept);
    }
    if (want_verdict) {
        if (use_dec)         // every row is the last row of its trace
            HIP_TRY(cs::launch_verdict(c.dtype, x, nullptr, w->final_norm, w->lm_head, va, B, B, d, c.rms_eps, dev_verdict_logits,
                                       dev_conf, dev_verdict, dev_accept, s));
        else if (prune)
            HIP_TRY(cs::launch_verdict(c.dtype, (const float *)(ws + L.x_last), nullptr, w->final_norm, w->lm_head, va, B, B, d,
                                       c.rms_eps, dev_verdict_logits, dev_conf, dev_verdict, dev_accept, s));
        else
            HIP_TRY(cs::launch_verdict(c.dtype, x, last_row, w->final_norm, w->lm_head, va, B, T, d, c.rms_eps,
                                       dev_verdict_logits, dev_conf, dev_verdict, dev_accept, s));
    }
    if (ex.head) {
        // Logits of the whole vocabulary at the last position of every trace: final norm of those B rows (two bf16
        // terms, so the operand carries ~16 mantissa bits), one GEMM against the head, then arg max / log-sum-exp.
        char *hs = (char *)ex.head_scratch;
        const float *xl = use_dec ? x : (const float *)(ws + L.x_last);
        if (!prune && !use_dec) {
            HIP_TRY(cs::launch_gather_rows(x, hs + HL.x, last_row, B, T, (size_t)d * 4, s));
            xl = (const float *)(hs + HL.x);
        }
        const bool bf = c.dtype == CONFSPEC_DTYPE_BF16;
        HIP_TRY(cs::launch_rmsnorm(c.dtype, xl, w->final_norm, hs + HL.y, B, d, c.rms_eps, bf ? 2 : 1, s));
        if (use_dec && d <= 64 * cs::DEC_MAX_KT && c.vocab % 16 == 0) {
            // generation step: the head streams once against the B rows, and every workgroup keeps only the running
            // (max, arg max, sum of exponentials) of its columns - the [B, vocab] logits are never written
            cs::DecGemm gh = {};
            gh.X = (const cs::bf16 *)(hs + HL.y); gh.ldx = 2 * d; gh.W = (const cs::bf16 *)w->lm_head; gh.M = B; gh.K = d;
            gh.n_ct = c.vocab / 16;
            cs::dec_gemm_plan(d, gh.n_ct, &gh.S, &gh.nwg);
            gh.head_part = (float *)(hs + HL.part);
            HIP_TRY(cs::launch_dec_gemm(gh, cs::DEC_EPI_HEAD, false, s));
            HIP_TRY(cs::launch_dec_head_final(gh.head_part, gh.nwg, B, want_verdict ? dev_verdict_logits : nullptr, va.n_verdict,
                                              ex.head->token, ex.head->max_logit, ex.head->lse,
                                              want_verdict ? ex.head->conf_full : nullptr, s));
            HIP_TRY(mark(CONFSPEC_PHASE_END));
            return CONFSPEC_OK;
        }
        if ((rc = run_gemm(ctx, hs + HL.y, w->lm_head, hs + HL.logits, B, c.vocab, d, cs::EPI_STORE_F32, bf ? 2 : 1, 1, s,
                           bf ? (float *)(ws + L.splitk) : nullptr, bf ? L.splitk_bytes : 0)))
            return rc;
        HIP_TRY(cs::launch_head_reduce((const float *)(hs + HL.logits), B, c.vocab, want_verdict ? dev_verdict_logits : nullptr,
                                       va.n_verdict, ex.head->token, ex.head->max_logit, ex.head->lse,
                                       want_verdict ? ex.head->conf_full : nullptr, s));
    }
    HIP_TRY(mark(CONFSPEC_PHASE_END));
    return CONFSPEC_OK;
}

int confspec_verify(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                    const confspec_batch *batch, const int32_t *h_verdict_ids, int32_t n_verdict,
                    const float *h_tau, int32_t n_tau, void *dev_workspace, size_t workspace_bytes,
                    float *dev_verdict_logits, float *dev_conf, int32_t *dev_verdict, uint8_t *dev_accept,
                    confspec_stream stream) {
    if (ctx && !h_verdict_ids) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids or tau pointer is null");
    return verify_impl(ctx, w, kv, batch, h_verdict_ids, n_verdict, h_tau, n_tau, dev_workspace, workspace_bytes,
                       dev_verdict_logits, dev_conf, dev_verdict, dev_accept, PassExtras{}, stream);
}

int confspec_verify_shared(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_group_start, const int32_t *h_group_start,
                           int32_t n_groups, const int32_t *h_verdict_ids, int32_t n_verdict, const float *h_tau,
                           int32_t n_tau, void *dev_workspace, size_t workspace_bytes, float *dev_verdict_logits,
                           float *dev_conf, int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!h_verdict_ids) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids or tau pointer is null");
    if (!dev_group_start || !h_group_start) return fail(ctx, CONFSPEC_E_INVALID_ARG, "group_start is null");
    PassExtras ex;
    ex.dev_group_start = dev_group_start;
    ex.h_group_start = h_group_start;
    ex.n_groups = n_groups;
    return verify_impl(ctx, w, kv, batch, h_verdict_ids, n_verdict, h_tau, n_tau, dev_workspace, workspace_bytes,
                       dev_verdict_logits, dev_conf, dev_verdict, dev_accept, ex, stream);
}

int confspec_verify_append(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_n_append, const int32_t *h_n_append,
                           const int32_t *h_verdict_ids, int32_t n_verdict, const float *h_tau, int32_t n_tau,
                           void *dev_workspace, size_t workspace_bytes, float *dev_verdict_logits, float *dev_conf,
                           int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!dev_n_append || !h_n_append) return fail(ctx, CONFSPEC_E_INVALID_ARG, "n_append is null");
    if (!h_verdict_ids) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids or tau pointer is null");
    PassExtras ex;
    ex.dev_n_append = dev_n_append;
    ex.h_n_append = h_n_append;
    return verify_impl(ctx, w, kv, batch, h_verdict_ids, n_verdict, h_tau, n_tau, dev_workspace, workspace_bytes,
                       dev_verdict_logits, dev_conf, dev_verdict, dev_accept, ex, stream);
}

// ---- the pass on the library's own scratch: no allocation anywhere on the way ----
namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on each device, looked up on the first call there

int static_scratch_ptr(confspec_ctx *ctx, void **out) {
    int dev = ctx->device;
    if (dev < 0 || dev >= MAX_DEVICES) return fail(ctx, CONFSPEC_E_UNSUPPORTED, "device %d: at most %d devices", dev, MAX_DEVICES);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;   // this device's copy of the array (the current device is ctx->device: checked by the caller)
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255)) return fail(ctx, CONFSPEC_E_HIP, "static scratch has address %p", p);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return CONFSPEC_OK;
}
}  // namespace

int confspec_static_scratch_need(const confspec_ctx *ctx, const confspec_batch *batch, size_t *out_bytes) {
    if (!ctx || !out_bytes) return CONFSPEC_E_INVALID_ARG;
    int rc;
    if ((rc = check_batch(ctx, batch, INT32_MAX, nullptr)) != CONFSPEC_OK) return rc;
    *out_bytes = ws_layout(ctx, batch->T, batch->B, batch).total;
    return CONFSPEC_OK;
}

int confspec_verify_static(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *h_verdict_ids, int32_t n_verdict,
                           const float *h_tau, int32_t n_tau, float *dev_verdict_logits, float *dev_conf,
                           int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!h_verdict_ids) return fail(ctx, CONFSPEC_E_INVALID_ARG, "verdict ids or tau pointer is null");
    int rc;
    size_t need = 0;
    if ((rc = confspec_static_scratch_need(ctx, batch, &need)) != CONFSPEC_OK) return rc;
    if (need > (size_t)CONFSPEC_STATIC_SCRATCH_BYTES)
        return fail(ctx, CONFSPEC_E_WORKSPACE,
                    "a batch of %d tokens in %d traces needs %zu bytes of scratch, the static array holds %zu; use "
                    "confspec_verify with a workspace",
                    batch->T, batch->B, need, (size_t)CONFSPEC_STATIC_SCRATCH_BYTES);
    if ((rc = check_device(ctx)) != CONFSPEC_OK) return rc;
    void *ptr = nullptr;
    if ((rc = static_scratch_ptr(ctx, &ptr)) != CONFSPEC_OK) return rc;
    // Nothing in the workspace has to start at zero: every slice is written by the pass before it is read (plans,
    // maps, activations, partial products), so the last call's contents are simply overwritten.
    PassExtras ex;
    ex.exact_layout = true;
    return verify_impl(ctx, w, kv, batch, h_verdict_ids, n_verdict, h_tau, n_tau, ptr, (size_t)CONFSPEC_STATIC_SCRATCH_BYTES,
                       dev_verdict_logits, dev_conf, dev_verdict, dev_accept, ex, stream);
}

size_t confspec_head_scratch_bytes(const confspec_ctx *ctx, int32_t max_B) {
    if (!ctx || max_B < 1) return 0;
    return head_layout(ctx->cfg, max_B).total;
}

int confspec_generate_step(confspec_ctx *ctx, const confspec_weights *w, const confspec_kv *kv,
                           const confspec_batch *batch, const int32_t *dev_n_append, const int32_t *h_n_append,
                           const int32_t *h_verdict_ids, int32_t n_verdict, void *dev_workspace, size_t workspace_bytes,
                           void *dev_head_scratch, size_t head_scratch_bytes, const confspec_head_out *out,
                           confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!out) return fail(ctx, CONFSPEC_E_INVALID_ARG, "out is null");
    if ((dev_n_append == nullptr) != (h_n_append == nullptr))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "dev_n_append and h_n_append must both be given or both be null");
    PassExtras ex;
    ex.dev_n_append = dev_n_append;
    ex.h_n_append = h_n_append;
    ex.head = out;
    ex.head_scratch = dev_head_scratch;
    ex.head_scratch_bytes = head_scratch_bytes;
    const float tau = 0.5f;   // the gate bit is not an output of this call
    return verify_impl(ctx, w, kv, batch, h_verdict_ids, n_verdict, &tau, 1, dev_workspace, workspace_bytes, nullptr, nullptr,
                       nullptr, nullptr, ex, stream);
}

// ---- single-step entry points ------------------------------------------------------------------
static int check_terms(confspec_ctx *ctx, int terms, const char *what) {
    if (terms != 1 && !((terms == 2 || terms == 3) && ctx->cfg.dtype == CONFSPEC_DTYPE_BF16))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "%s must be 1, or 2 / 3 for a bf16 context (got %d)", what, terms);
    return CONFSPEC_OK;
}

int confspec_op_gemm(confspec_ctx *ctx, const void *dev_A, const void *dev_W, void *dev_out, int32_t M, int32_t N,
                     int32_t K, int32_t epilogue, int32_t a_terms, int32_t out_terms, void *dev_scratch,
                     size_t scratch_bytes, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!dev_A || !dev_W || !dev_out) return fail(ctx, CONFSPEC_E_INVALID_ARG, "null operand");
    if (dev_scratch && ((uintptr_t)dev_scratch & 15)) return fail(ctx, CONFSPEC_E_WORKSPACE, "scratch is not 16-byte aligned");
    if (((uintptr_t)dev_A | (uintptr_t)dev_W | (uintptr_t)dev_out) & 15)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "operands must be 16-byte aligned");
    if (M < 1 || N < 1 || K < 1) return fail(ctx, CONFSPEC_E_INVALID_ARG, "M, N, K must be >= 1");
    if (epilogue < 0 || epilogue > 2) return fail(ctx, CONFSPEC_E_INVALID_ARG, "unknown epilogue %d", epilogue);
    int rc;
    if ((rc = check_terms(ctx, a_terms, "a_terms")) || (rc = check_terms(ctx, out_terms, "out_terms"))) return rc;
    if (out_terms != 1 && epilogue != CONFSPEC_EPI_SWIGLU)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "out_terms != 1 needs the SwiGLU epilogue");
    if (ctx->cfg.dtype == CONFSPEC_DTYPE_BF16) {
        if (N % 128 || K % 64) return fail(ctx, CONFSPEC_E_UNSUPPORTED, "bf16 GEMM needs N %% 128 == 0 and K %% 64 == 0");
    } else if (N % 64 || K % 16) {
        return fail(ctx, CONFSPEC_E_UNSUPPORTED, "fp32 GEMM needs N %% 64 == 0 and K %% 16 == 0");
    }
    if ((rc = check_device(ctx))) return rc;
    return run_gemm(ctx, dev_A, dev_W, dev_out, M, N, K, epilogue, a_terms, out_terms, (hipStream_t)stream,
                    (float *)dev_scratch, dev_scratch ? scratch_bytes : 0);
}

size_t confspec_op_gemm_scratch_bytes(const confspec_ctx *ctx, int32_t M, int32_t N, int32_t K, int32_t a_terms) {
    if (!ctx || ctx->cfg.dtype != CONFSPEC_DTYPE_BF16 || M < 1 || N < 1 || K < 1 || a_terms < 1 || a_terms > 3) return 0;
    return cs::gemm_splitk_bytes(ctx->set.gemm, M, N, K * (a_terms == 2 ? 2 : 1));
}

int confspec_op_rmsnorm(confspec_ctx *ctx, const float *dev_x, const void *dev_g, void *dev_out, int32_t n_rows,
                        int32_t out_terms, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!dev_x || !dev_g || !dev_out || n_rows < 1) return fail(ctx, CONFSPEC_E_INVALID_ARG, "bad argument");
    int rc;
    if ((rc = check_terms(ctx, out_terms, "out_terms"))) return rc;
    if ((rc = check_device(ctx))) return rc;
    HIP_TRY(cs::launch_rmsnorm(ctx->cfg.dtype, dev_x, dev_g, dev_out, n_rows, ctx->cfg.d_model, ctx->cfg.rms_eps,
                               out_terms, (hipStream_t)stream));
    return CONFSPEC_OK;
}

static int check_lo(confspec_ctx *ctx, const void *a, const void *b, const void *c3) {
    int n = (a != nullptr) + (b != nullptr) + (c3 != nullptr);
    if (n != 0 && n != 3) return fail(ctx, CONFSPEC_E_INVALID_ARG, "second-term pointers must be all set or all null");
    if (n == 3 && ctx->cfg.dtype != CONFSPEC_DTYPE_BF16)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "second-term operands need a bf16 context");
    return CONFSPEC_OK;
}

int confspec_op_rope_split(confspec_ctx *ctx, const confspec_batch *batch, int32_t max_prefix_len,
                           const float *dev_qkv, void *dev_q, void *dev_k, void *dev_v, void *dev_q_lo,
                           void *dev_k_lo, void *dev_v_lo, void *dev_workspace, size_t workspace_bytes,
                           confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!dev_qkv || !dev_q || !dev_k || !dev_v) return fail(ctx, CONFSPEC_E_INVALID_ARG, "null operand");
    if (int rl = check_lo(ctx, dev_q_lo, dev_k_lo, dev_v_lo)) return rl;
    int rc, max_L = 0;
    if ((rc = check_batch(ctx, batch, max_prefix_len, &max_L)) != CONFSPEC_OK) return rc;
    const confspec_model_cfg &c = ctx->cfg;
    WsLayout L = ws_layout(ctx, batch->T, batch->B);
    if ((rc = check_ws(ctx, dev_workspace, workspace_bytes, L.total)) != CONFSPEC_OK) return rc;
    char *ws = (char *)dev_workspace;
    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(cs::launch_prep(batch->cu_suffix, batch->prefix_lens, batch->B, batch->T, max_L, (int32_t *)(ws + L.tok_trace),
                            (int32_t *)(ws + L.tok_pos), (int32_t *)(ws + L.last_row), s));
    HIP_TRY(cs::launch_rope_table((const int32_t *)(ws + L.tok_pos), batch->T, c.head_dim, c.rope_theta,
                                  (float *)(ws + L.rope_cos), (float *)(ws + L.rope_sin), s));
    HIP_TRY(cs::launch_rope_split(c.dtype, dev_qkv, (const float *)(ws + L.rope_cos), (const float *)(ws + L.rope_sin),
                                  dev_q, dev_k, dev_v, dev_q_lo, dev_k_lo, dev_v_lo, batch->T, c.n_q_heads, c.n_kv_heads,
                                  c.head_dim, s));
    return CONFSPEC_OK;
}

int confspec_op_qkv_rope(confspec_ctx *ctx, const confspec_batch *batch, int32_t max_prefix_len, const void *dev_h,
                         int32_t a_terms, const void *dev_wqkv_perm, void *dev_q, void *dev_k, void *dev_v,
                         void *dev_q_lo, void *dev_k_lo, void *dev_v_lo, void *dev_workspace, size_t workspace_bytes,
                         confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    const confspec_model_cfg &c = ctx->cfg;
    if (c.dtype != CONFSPEC_DTYPE_BF16 || c.head_dim != 128)
        return fail(ctx, CONFSPEC_E_UNSUPPORTED, "the rotating projection kernel needs a bf16 context with head_dim 128");
    if (!dev_h || !dev_wqkv_perm || !dev_q || !dev_k || !dev_v) return fail(ctx, CONFSPEC_E_INVALID_ARG, "null operand");
    if (int rl = check_lo(ctx, dev_q_lo, dev_k_lo, dev_v_lo)) return rl;
    int rc, max_L = 0;
    if ((rc = check_terms(ctx, a_terms, "a_terms"))) return rc;
    if ((rc = check_batch(ctx, batch, max_prefix_len, &max_L)) != CONFSPEC_OK) return rc;
    WsLayout L = ws_layout(ctx, batch->T, batch->B);
    if ((rc = check_ws(ctx, dev_workspace, workspace_bytes, L.total)) != CONFSPEC_OK) return rc;
    char *ws = (char *)dev_workspace;
    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(cs::launch_prep(batch->cu_suffix, batch->prefix_lens, batch->B, batch->T, max_L, (int32_t *)(ws + L.tok_trace),
                            (int32_t *)(ws + L.tok_pos), (int32_t *)(ws + L.last_row), s));
    HIP_TRY(cs::launch_rope_table((const int32_t *)(ws + L.tok_pos), batch->T, c.head_dim, c.rope_theta,
                                  (float *)(ws + L.rope_cos), (float *)(ws + L.rope_sin), s));
    cs::RopeArgs ra = {(const float *)(ws + L.rope_cos), (const float *)(ws + L.rope_sin), dev_q, dev_k, dev_v,
                       dev_q_lo, dev_k_lo, dev_v_lo, c.n_q_heads, c.n_kv_heads};
    HIP_TRY(cs::launch_gemm_bf16_rope(ctx->set.gemm, (const cs::bf16 *)dev_h, (const cs::bf16 *)dev_wqkv_perm, batch->T,
                                      (c.n_q_heads + 2 * c.n_kv_heads) * c.head_dim, c.d_model, a_terms, ra,
                                      (float *)(ws + L.splitk), L.splitk_bytes, s));
    return CONFSPEC_OK;
}

int confspec_op_attention(confspec_ctx *ctx, const confspec_kv *kv, const confspec_batch *batch, int32_t layer,
                          const void *dev_q, const void *dev_k_suffix, const void *dev_v_suffix, const void *dev_q_lo,
                          const void *dev_k_lo, const void *dev_v_lo, void *dev_out, int32_t out_terms,
                          void *dev_workspace, size_t workspace_bytes, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (int rl = check_lo(ctx, dev_q_lo, dev_k_lo, dev_v_lo)) return rl;
    if (int rt = check_terms(ctx, out_terms, "out_terms")) return rt;
    if (!dev_q || !dev_k_suffix || !dev_v_suffix || !dev_out) return fail(ctx, CONFSPEC_E_INVALID_ARG, "null operand");
    if (!kv) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv is null");
    if (layer < 0 || layer >= (ctx->cfg.n_layers > 0 ? ctx->cfg.n_layers : 1))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "layer %d out of range", layer);
    int rc, max_L = 0;
    if ((rc = check_batch(ctx, batch, (int64_t)kv->max_blocks_per_seq * kv->block_size, &max_L)) != CONFSPEC_OK) return rc;
    if ((rc = check_kv(ctx, kv, max_L > 0)) != CONFSPEC_OK) return rc;
    WsLayout L = ws_layout(ctx, batch->T, batch->B);
    if ((rc = check_ws(ctx, dev_workspace, workspace_bytes, L.total)) != CONFSPEC_OK) return rc;
    char *ws = (char *)dev_workspace;
    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    cs::AttnPlanCounts pc;
    if ((rc = run_plan(ctx, batch, Groups{}, max_L, ws, L, &pc, s)) != CONFSPEC_OK) return rc;
    cs::AttnArgs a = make_attn_args(ctx->cfg, kv, batch, (const int32_t *)(ws + L.tok_trace), layer, dev_q, dev_k_suffix, dev_v_suffix, dev_q_lo, dev_k_lo,
                                    dev_v_lo, dev_out, out_terms);
    return run_attention(ctx, a, ws, L, pc, false, s);
}

int confspec_op_verdict_gate(confspec_ctx *ctx, const confspec_batch *batch, const float *dev_x,
                             const void *dev_final_norm, const void *dev_lm_head, const int32_t *h_verdict_ids,
                             int32_t n_verdict, const float *h_tau, int32_t n_tau, void *dev_workspace,
                             size_t workspace_bytes, float *dev_verdict_logits, float *dev_conf,
                             int32_t *dev_verdict, uint8_t *dev_accept, confspec_stream stream) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!dev_x || !dev_final_norm || !dev_lm_head || !dev_verdict_logits || !dev_conf || !dev_verdict || !dev_accept)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "null operand");
    int rc, max_L = 0;
    if ((rc = check_batch(ctx, batch, INT32_MAX, &max_L)) != CONFSPEC_OK) return rc;
    cs::VerdictArgs va;
    if ((rc = check_verdict(ctx, h_verdict_ids, n_verdict, h_tau, n_tau, &va)) != CONFSPEC_OK) return rc;
    const confspec_model_cfg &c = ctx->cfg;
    WsLayout L = ws_layout(ctx, batch->T, batch->B);
    if ((rc = check_ws(ctx, dev_workspace, workspace_bytes, L.total)) != CONFSPEC_OK) return rc;
    char *ws = (char *)dev_workspace;
    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    HIP_TRY(cs::launch_prep(batch->cu_suffix, batch->prefix_lens, batch->B, batch->T, max_L, (int32_t *)(ws + L.tok_trace),
                            (int32_t *)(ws + L.tok_pos), (int32_t *)(ws + L.last_row), s));
    HIP_TRY(cs::launch_verdict(c.dtype, dev_x, (const int32_t *)(ws + L.last_row), dev_final_norm, dev_lm_head, va,
                               batch->B, batch->T, c.d_model, c.rms_eps, dev_verdict_logits, dev_conf, dev_verdict,
                               dev_accept, s));
    return CONFSPEC_OK;
}

int confspec_op_workspace_slices(const confspec_ctx *ctx, int32_t T, int32_t B, const confspec_batch *exact, size_t *h_offsets,
                                 size_t *h_bytes, int32_t *n, size_t *total) {
    if (!ctx || !h_offsets || !h_bytes || !n || !total) return CONFSPEC_E_INVALID_ARG;
    if (T < 1 || B < 1) return fail(ctx, CONFSPEC_E_INVALID_ARG, "T and B must be >= 1");
    int rc;
    if (exact && (rc = check_batch(ctx, exact, INT32_MAX, nullptr)) != CONFSPEC_OK) return rc;
    if (exact && (exact->T != T || exact->B != B)) return fail(ctx, CONFSPEC_E_INVALID_ARG, "exact batch has other T / B");
    WsLayout L = ws_layout(ctx, T, B, exact);
    if (*n < L.n_slices) return fail(ctx, CONFSPEC_E_WORKSPACE, "%d slices, room for %d", L.n_slices, *n);
    for (int i = 0; i < L.n_slices; ++i) { h_offsets[i] = L.slice_off[i]; h_bytes[i] = L.slice_len[i]; }
    *n = L.n_slices;
    *total = L.total;
    return CONFSPEC_OK;
}

int confspec_phase_timing(confspec_ctx *ctx, int32_t enable) {
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    PhaseTimer &t = ctx->timer;
    if (enable && t.events.empty()) {
        int rc;
        if ((rc = check_device(ctx)) != CONFSPEC_OK) return rc;
        constexpr int N_EVENTS = 2048;     // a pass of 200 layers records fewer
        t.events.reserve(N_EVENTS);
        for (int i = 0; i < N_EVENTS; ++i) {
            hipEvent_t e;
            HIP_TRY(hipEventCreate(&e));
            t.events.push_back(e);
        }
        t.phase.assign(N_EVENTS, CONFSPEC_PHASE_OTHER);
    }
    t.enabled = enable != 0;
    t.used = 0;
    return CONFSPEC_OK;
}

int confspec_phase_times(confspec_ctx *ctx, float *h_ms, int32_t *h_intervals) {
    if (!ctx || !h_ms) return CONFSPEC_E_INVALID_ARG;
    PhaseTimer &t = ctx->timer;
    if (t.used < 2) return fail(ctx, CONFSPEC_E_INVALID_ARG, "no pass has been timed on this context");
    if (t.overflow) return fail(ctx, CONFSPEC_E_UNSUPPORTED, "the pass changed phase more often than there are events");
    for (int p = 0; p < CONFSPEC_N_PHASES; ++p) {
        h_ms[p] = 0.f;
        if (h_intervals) h_intervals[p] = 0;
    }
    HIP_TRY(hipEventSynchronize(t.events[t.used - 1]));
    for (int i = 0; i + 1 < t.used; ++i) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, t.events[i], t.events[i + 1]));
        int p = t.phase[i];
        if (p < 0 || p >= CONFSPEC_N_PHASES) continue;
        h_ms[p] += ms;
        if (h_intervals) h_intervals[p] += 1;
    }
    return CONFSPEC_OK;
}

int confspec_tune(confspec_ctx *ctx, const char *key, int32_t value) {
    if (!key) return CONFSPEC_E_INVALID_ARG;
    Settings &st = ctx ? ctx->set : g_default_settings;
    struct Entry { const char *key; int *field; int lo, hi; };
    const Entry table[] = {
        {"gemm_tile", &st.gemm.tile, 0, 7},
        {"gemm_group_m", &st.gemm.group_m, 0, 65536},
        {"gemm_splitk", &st.gemm.splitk, 0, 64},
        {"gemm_short_tile", &st.gemm.short_tile, 0, 1},
        {"split_layers", &st.split_layers, -1, 4096},
        {"prefetch_down", &st.prefetch_down, 0, 1},
        {"fuse_rope", &st.fuse_rope, 0, 1},
        {"decode_kernels", &st.decode_kernels, 0, 2},
        {"first_layers_f16", &st.first_layers_f16, 0, 1},
        {"prune_last_layer", &st.prune_last_layer, 0, 1},
        {"attn_precise_layers", &st.attn_precise_layers, 0, 4096},
        {"attn_target_items", &st.attn.target_items, 1, 65536},
        {"attn_split", &st.attn.force_split, 0, 5},
        {"attn_min_chunks", &st.attn.min_chunks, 1, 4096},
        {"attn_kernel", &st.attn.kernel, 0, 2},
    };
    for (const Entry &e : table)
        if (!strcmp(key, e.key)) {
            if (value < e.lo || value > e.hi) return CONFSPEC_E_INVALID_ARG;
            if (e.field == &st.gemm.tile && value != 0 && value != 1 && value != 4 && value != 7) return CONFSPEC_E_INVALID_ARG;
            *e.field = value;
            return CONFSPEC_OK;
        }
    return CONFSPEC_E_INVALID_ARG;
}

// ---- two-tier cascade (Section 4.2, Eq. 4; Algorithm 1, Stage 2) ----

namespace {
struct CascadeLayout {
    size_t keep, open_flag, pos_of, sel_idx, cu_out, plens_out, n_out, ids_out, table_out, logits_d, logits_t, conf_t, verdict_t,
        accept_t, total;
};
CascadeLayout cascade_layout(int64_t B, int64_t T, int64_t max_blocks) {
    CascadeLayout L;
    size_t at = 0;
    auto take = [&](size_t bytes) { size_t o = at; at += (bytes + 255) & ~(size_t)255; return o; };
    L.keep = take(B);
    L.open_flag = take(B);
    L.pos_of = take(B * 4);
    L.sel_idx = take(B * 4);
    L.cu_out = take((B + 1) * 4);
    L.plens_out = take(B * 4);
    L.n_out = take(8);
    L.ids_out = take(T * 4);
    L.table_out = take(B * max_blocks * 4);
    L.logits_d = take(B * CONFSPEC_MAX_VERDICT * 4);
    L.logits_t = take(B * CONFSPEC_MAX_VERDICT * 4);
    L.conf_t = take(B * 4);
    L.verdict_t = take(B * 4);
    L.accept_t = take(B);
    L.total = at;
    return L;
}
}  // namespace

size_t confspec_cascade_scratch_bytes(int32_t max_B, int32_t max_T, int32_t max_blocks_per_seq_target) {
    if (max_B < 1 || max_T < 1 || max_blocks_per_seq_target < 1) return 0;
    return cascade_layout(max_B, max_T, max_blocks_per_seq_target).total;
}

int confspec_cascade(confspec_ctx *draft, const confspec_weights *wd, const confspec_kv *kvd, void *ws_d, size_t ws_d_bytes,
                     confspec_ctx *target, const confspec_weights *wt, const confspec_kv *kvt, void *ws_t,
                     size_t ws_t_bytes, const confspec_batch *batch, const confspec_requests *req,
                     const int32_t *h_verdict_ids, int32_t n_verdict, float gamma, void *dev_scratch, size_t scratch_bytes,
                     const confspec_cascade_out *out, int32_t *h_n_target, confspec_stream stream) {
    confspec_ctx *ctx = draft;
    if (!ctx) return CONFSPEC_E_INVALID_ARG;
    if (!target) return fail(ctx, CONFSPEC_E_INVALID_ARG, "target context is null");
    for (int i = 0; h_verdict_ids && i < n_verdict && i < CONFSPEC_MAX_VERDICT; ++i)
        if (h_verdict_ids[i] < 0 || h_verdict_ids[i] >= std::min(draft->cfg.vocab, target->cfg.vocab))
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "verdict id %d = %d outside the smaller vocabulary [0, %d)", i,
                        h_verdict_ids[i], std::min(draft->cfg.vocab, target->cfg.vocab));
    if (!out || !out->conf_draft || !out->verdict_draft || !out->conf_target || !out->verdict_target || !out->decision ||
        !out->escalated || !out->target_ran || !out->accepted_steps)
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "an output pointer is null");
    if (!(gamma >= 0.0f)) return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "gamma = %g is negative or not a number", (double)gamma);
    int rc, max_L = 0;
    if (!kvd || !kvt) return fail(ctx, CONFSPEC_E_INVALID_ARG, "kv is null");
    int64_t cap_d = (int64_t)kvd->max_blocks_per_seq * kvd->block_size, cap_t = (int64_t)kvt->max_blocks_per_seq * kvt->block_size;
    if ((rc = check_batch(ctx, batch, std::min(cap_d, cap_t), &max_L)) != CONFSPEC_OK) return rc;
    if ((rc = check_kv(ctx, kvd, max_L > 0)) != CONFSPEC_OK) return rc;
    if ((rc = check_kv(target, kvt, max_L > 0)) != CONFSPEC_OK) return fail(ctx, rc, "target: %s", target->err.c_str());
    const int B = batch->B, T = batch->T;
    if (!req || !req->req_start || !req->h_req_start) return fail(ctx, CONFSPEC_E_INVALID_ARG, "requests or one of its arrays is null");
    const int R = req->n_requests;
    if (R < 1 || R > B) return fail(ctx, CONFSPEC_E_INVALID_ARG, "n_requests = %d outside [1, B = %d]", R, B);
    if (req->h_req_start[0] != 0 || req->h_req_start[R] != B)
        return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "req_start must run from 0 to B = %d (got %d .. %d)", B, req->h_req_start[0],
                    req->h_req_start[R]);
    for (int r = 0; r < R; ++r)
        if (req->h_req_start[r + 1] <= req->h_req_start[r])
            return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "req_start not strictly increasing at request %d (every request needs >= 1 step)", r);
    if ((req->parent == nullptr) != (req->h_parent == nullptr))
        return fail(ctx, CONFSPEC_E_INVALID_ARG, "parent and h_parent must both be given or both be null");
    for (int r = 0; req->h_parent && r < R; ++r)
        for (int b = req->h_req_start[r]; b < req->h_req_start[r + 1]; ++b)
            if (req->h_parent[b] != -1 && (req->h_parent[b] < req->h_req_start[r] || req->h_parent[b] >= b))
                return fail(ctx, CONFSPEC_E_OUT_OF_RANGE, "parent[%d] = %d: must be -1 or an earlier trace of the same request", b,
                            req->h_parent[b]);
    CascadeLayout C = cascade_layout(B, T, kvt->max_blocks_per_seq);
    if ((rc = check_ws(ctx, dev_scratch, scratch_bytes, C.total)) != CONFSPEC_OK) return rc;
    // the large model's pass is a sub-batch of this one, so a workspace for the whole batch is enough for it
    if ((rc = check_ws(ctx, ws_t, ws_t_bytes, ws_layout(target, T, B).total)) != CONFSPEC_OK) return rc;
    if (!wt || wt->packed != 1) return fail(ctx, CONFSPEC_E_INVALID_ARG, "target weights must be packed with confspec_pack_weights");

    if (int rd = check_device(ctx)) return rd;
    hipStream_t s = (hipStream_t)stream;
    char *sc = (char *)dev_scratch;
    uint8_t *keep = (uint8_t *)(sc + C.keep);
    int32_t *pos_of = (int32_t *)(sc + C.pos_of), *sel_idx = (int32_t *)(sc + C.sel_idx);
    int32_t *cu_out = (int32_t *)(sc + C.cu_out), *plens_out = (int32_t *)(sc + C.plens_out), *n_out = (int32_t *)(sc + C.n_out);
    int32_t *ids_out = (int32_t *)(sc + C.ids_out), *table_out = (int32_t *)(sc + C.table_out);
    float *conf_t_c = (float *)(sc + C.conf_t);
    int32_t *verdict_t_c = (int32_t *)(sc + C.verdict_t);

    // small model on every trace; its gate bit conf >= gamma is taken in the verdict kernel.  Thresholds above 1
    // keep nothing, which is what any value above 1 means.
    float tau = gamma > 1.0f ? 1.0f : gamma;
    const bool keep_nothing = gamma > 1.0f;
    if ((rc = confspec_verify(draft, wd, kvd, batch, h_verdict_ids, n_verdict, &tau, 1, ws_d, ws_d_bytes,
                              (float *)(sc + C.logits_d), out->conf_draft, out->verdict_draft, keep, s)) != CONFSPEC_OK)
        return rc;
    if (keep_nothing) HIP_TRY(hipMemsetAsync(keep, 0, B, s));
    HIP_TRY(cs::launch_cascade_select(keep, out->verdict_draft, req->req_start, req->parent, R, B, batch->cu_suffix,
                                      batch->prefix_lens, T, (uint8_t *)(sc + C.open_flag), out->target_ran, pos_of, sel_idx,
                                      cu_out, plens_out, n_out, s));
    HIP_TRY(cs::launch_cascade_gather(pos_of, batch->cu_suffix, cu_out, batch->suffix_ids, ids_out, kvt->block_table,
                                      table_out, kvt->max_blocks_per_seq, B, T, s));
    // The one host round trip of the call: how many traces the large model sees, their suffix offsets and prefix
    // lengths (the host plans that pass's launches from them).
    int32_t h_n[2] = {0, 0};
    std::vector<int32_t> h_cu(B + 1), h_pl(B);
    HIP_TRY(hipMemcpyAsync(h_n, n_out, sizeof h_n, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_cu.data(), cu_out, (size_t)(B + 1) * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipMemcpyAsync(h_pl.data(), plens_out, (size_t)B * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(hipStreamSynchronize(s));
    const int n = h_n[0];
    if (n < 0 || n > B || h_n[1] < 0 || h_n[1] > T) return fail(ctx, CONFSPEC_E_HIP, "selection returned %d traces, %d tokens", n, h_n[1]);
    if (h_n_target) *h_n_target = n;
    if (n > 0) {
        confspec_batch sub = {n, h_n[1], ids_out, cu_out, plens_out, h_cu.data(), h_pl.data()};
        confspec_kv kv_sub = *kvt;
        kv_sub.block_table = table_out;
        if ((rc = confspec_verify(target, wt, &kv_sub, &sub, h_verdict_ids, n_verdict, &tau, 1, ws_t, ws_t_bytes,
                                  (float *)(sc + C.logits_t), conf_t_c, verdict_t_c, (uint8_t *)(sc + C.accept_t), s)) !=
            CONFSPEC_OK)
            return fail(ctx, rc, "target: %s", target->err.c_str());
    }
    HIP_TRY(cs::launch_cascade_merge(keep, out->verdict_draft, out->conf_draft, pos_of, conf_t_c, verdict_t_c, req->req_start,
                                     req->parent, R, B, n, out->conf_target, out->verdict_target, out->decision,
                                     out->escalated, out->selected, out->conf_used, out->accepted_steps, s));
    return CONFSPEC_OK;
}

}  // extern "C"
