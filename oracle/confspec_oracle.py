"""fp64 CPU oracle for the batched verification pass (TEST INFRASTRUCTURE).

This file is the slow, plain definition that the GPU library is checked
against.  It is imported only by the tests, the smoke check and the benchmark's
CPU-baseline leg; the product path never calls it and shares no code with it.

What it computes, and where the paper defines it:

* A verifier model reads the cached reasoning context, the drafted step, the
  target's step and a verification prompt, and emits a decision token together
  with that token's softmax probability (Section 4.2, Eq. 2 and Eq. 3, and the
  sentence after Eq. 3 on the "Yes"/"No" verification token).
* The probability that counts is the one of the *predicted* decision
  (Section 4.1, "Confidence as a Reliability Signal").
* The decision is kept when that probability is at least the threshold gamma
  and escalated to the larger model otherwise (Section 4.2, Eq. 4; Algorithm 1,
  the statement that assigns V inside the verification loop).

The paper does not spell out the transformer under the verifier; it is the
standard pre-norm decoder its model families use (RMSNorm, rotary positions in
the half-split pairing, grouped-query causal attention, SwiGLU MLP, no biases).
Readings taken where the paper is silent: the softmax runs over the verdict
tokens only, so their probabilities sum to one; ties in the argmax go to the
lowest index; cached keys are stored after rotation; the suffix is never
written back to the cache.

Every function works on float64 numpy arrays.  Nothing is blocked, fused or
reordered beyond the formulas as written.
"""
from __future__ import annotations

import math
from typing import Callable, List, Optional, Sequence

import numpy as np


# --------------------------------------------------------------------------- #
# decoder building blocks (standard definitions)
# --------------------------------------------------------------------------- #
def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """RMSNorm(x)_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i, over the last axis."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(a: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split pairing (i, i + hd/2).

    a: [n, H, hd]; pos: [n] absolute positions.  For i in [0, hd/2):
    phi = pos * theta^(-2i/hd);
    (a_i, a_{i+hd/2}) <- (a_i cos phi - a_{i+hd/2} sin phi, a_{i+hd/2} cos phi + a_i sin phi).
    """
    hd = a.shape[-1]
    half = hd // 2
    i = np.arange(half, dtype=np.float64)
    inv_freq = theta ** (-2.0 * i / hd)
    phi = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]
    c = np.cos(phi)[:, None, :]
    s = np.sin(phi)[:, None, :]
    lo, hi = a[..., :half], a[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax(s: np.ndarray, axis: int = -1) -> np.ndarray:
    m = np.max(s, axis=axis, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=axis, keepdims=True)


def attention(q: np.ndarray, k_all: np.ndarray, v_all: np.ndarray, L: int) -> np.ndarray:
    """Grouped-query causal attention of S new rows over L cached + S new keys.

    q: [S, Hq, hd]; k_all, v_all: [L + S, Hkv, hd].  Row t (absolute position
    L + t) sees keys j <= L + t.  Query head i reads kv head i // (Hq / Hkv).
    """
    S, Hq, hd = q.shape
    Hkv = k_all.shape[1]
    G = Hq // Hkv
    n = k_all.shape[0]
    visible = np.arange(n)[None, :] <= (L + np.arange(S))[:, None]
    out = np.empty_like(q)
    for i in range(Hq):
        c = i // G
        s = q[:, i, :] @ k_all[:, c, :].T / math.sqrt(hd)
        s = np.where(visible, s, -np.inf)
        p = softmax(s, axis=-1)
        out[:, i, :] = p @ v_all[:, c, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def decoder_layer(x: np.ndarray, pos: np.ndarray, lw: dict, k_prefix: np.ndarray,
                  v_prefix: np.ndarray, cfg):
    """One pre-norm decoder layer on S new rows placed after L cached rows.

    x: [S, d]; pos: [S]; k_prefix, v_prefix: [L, Hkv, hd] (keys already rotated).
    Returns (x_out, k_new, v_new) with k_new, v_new: [S, Hkv, hd] (k_new rotated).
    """
    S = x.shape[0]
    L = k_prefix.shape[0]
    hd = cfg.head_dim
    h = rmsnorm(x, lw["attn_norm"], cfg.rms_eps)
    q = (h @ lw["wq"].T).reshape(S, cfg.n_q_heads, hd)
    k = (h @ lw["wk"].T).reshape(S, cfg.n_kv_heads, hd)
    v = (h @ lw["wv"].T).reshape(S, cfg.n_kv_heads, hd)
    q = rope(q, pos, cfg.rope_theta)
    k = rope(k, pos, cfg.rope_theta)
    k_all = np.concatenate([k_prefix, k], axis=0)
    v_all = np.concatenate([v_prefix, v], axis=0)
    o = attention(q, k_all, v_all, L).reshape(S, cfg.n_q_heads * hd)
    x = x + o @ lw["wo"].T
    h2 = rmsnorm(x, lw["mlp_norm"], cfg.rms_eps)
    x = x + (silu(h2 @ lw["wg"].T) * (h2 @ lw["wu"].T)) @ lw["wd"].T
    return x, k, v


def gather_prefix(blocks: np.ndarray, L: int) -> np.ndarray:
    """Dense [L, Hkv, hd] rows from the trace's physical blocks, in logical order.

    blocks: [n, Hkv, block_size, hd], block i holding logical rows
    i*block_size .. i*block_size + block_size - 1 of the trace: logical row j
    lives in blocks[j // block_size][:, j % block_size, :].
    """
    n, Hkv, bs, hd = blocks.shape
    rows = np.empty((L, Hkv, hd), dtype=np.float64)
    for j in range(L):
        rows[j] = blocks[j // bs, :, j % bs, :]
    return rows


# --------------------------------------------------------------------------- #
# the pass
# --------------------------------------------------------------------------- #
def forward(cfg, model, traces: Sequence[dict], keep_kv: bool = False):
    """Run every trace's new tokens through all layers.

    model: object with embed_rows(ids), layer(l) -> dict of float64 matrices.
    Each trace is a dict with
      ids      : int array [S] new token ids (placed at positions L .. L+S-1)
      L        : cached prefix length
      k_prefix : callable l -> [L, Hkv, hd] float64 (rotated keys), same for v_prefix
    Returns (xs, kvs): xs[b] = [S_b, d] residual stream after the last layer;
    kvs[b][l] = (k_new, v_new) if keep_kv else None.

    Layers are the outer loop only so that each layer's matrices are widened to
    float64 once; no trace ever reads another trace's data.
    """
    xs, poss = [], []
    for tr in traces:
        ids = np.asarray(tr["ids"], dtype=np.int64)
        xs.append(np.asarray(model.embed_rows(ids), dtype=np.float64))
        poss.append(tr["L"] + np.arange(len(ids)))
    kvs = [[None] * cfg.n_layers for _ in traces]
    for l in range(cfg.n_layers):
        lw = model.layer(l)
        for b, tr in enumerate(traces):
            if xs[b].shape[0] == 0:       # a trace with no new tokens has nothing to compute
                if keep_kv:
                    kvs[b][l] = (np.zeros((0, cfg.n_kv_heads, cfg.head_dim)),) * 2
                continue
            kp = np.asarray(tr["k_prefix"](l), dtype=np.float64)
            vp = np.asarray(tr["v_prefix"](l), dtype=np.float64)
            xs[b], k_new, v_new = decoder_layer(xs[b], poss[b], lw, kp, vp, cfg)
            if keep_kv:
                kvs[b][l] = (k_new, v_new)
    return xs, kvs


def verdict_logits(x_last: np.ndarray, final_norm: np.ndarray, lm_rows: np.ndarray,
                   eps: float) -> np.ndarray:
    """z_v = RMSNorm(x_last) . W_lm[verdict_ids[v]] (Section 4.2: the verifier's
    decision is read as a verification token at the last position)."""
    y = rmsnorm(x_last, final_norm, eps)
    return lm_rows @ y


def confidence(z: np.ndarray):
    """(p, r, conf): softmax over the verdict logits, the predicted decision
    r = argmax (lowest index on ties) and its probability (Eq. 3; Section 4.1)."""
    p = softmax(np.asarray(z, dtype=np.float64), axis=-1)
    r = int(np.argmax(p))
    return p, r, float(p[r])


def gate(conf: np.ndarray, taus: Sequence[float]) -> np.ndarray:
    """accept[i, b] = 1 iff conf[b] >= taus[i] (Eq. 4: keep the verifier's own
    decision); 0 means escalate to the larger model."""
    conf = np.asarray(conf, dtype=np.float64)
    return np.stack([(conf >= float(t)) for t in taus]).astype(np.uint8)


def verify(cfg, model, kv, block_size: int, suffix_ids, cu_suffix, prefix_lens,
           verdict_ids, taus, trace_subset: Optional[Sequence[int]] = None) -> dict:
    """The whole pass for traces in `trace_subset` (default: all).

    kv: object with block_table [B, max_blocks] and k_blocks(l, ids), v_blocks(l, ids)
    returning [n, Hkv, block_size, hd] float64.
    Returns dict(logits [n, n_verdict], probs, conf [n], verdict [n], accept [n_tau, n]).
    """
    suffix_ids = np.asarray(suffix_ids)
    cu = np.asarray(cu_suffix, dtype=np.int64)
    Ls = np.asarray(prefix_lens, dtype=np.int64)
    B = len(Ls)
    which = list(range(B)) if trace_subset is None else list(trace_subset)
    traces = []
    for b in which:
        L = int(Ls[b])
        nblk = (L + block_size - 1) // block_size
        blk_ids = np.asarray(kv.block_table[b][:nblk], dtype=np.int64)

        def k_prefix(l, blk_ids=blk_ids, L=L):
            if L == 0:
                return np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
            return gather_prefix(kv.k_blocks(l, blk_ids), L)

        def v_prefix(l, blk_ids=blk_ids, L=L):
            if L == 0:
                return np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
            return gather_prefix(kv.v_blocks(l, blk_ids), L)

        traces.append(dict(ids=suffix_ids[cu[b]:cu[b + 1]], L=L, k_prefix=k_prefix, v_prefix=v_prefix))
    xs, _ = forward(cfg, model, traces)
    g = np.asarray(model.final_norm, dtype=np.float64)
    lm_rows = np.asarray(model.lm_head_rows(np.asarray(verdict_ids)), dtype=np.float64)
    logits, probs, verdict, conf = [], [], [], []
    for x in xs:
        z = verdict_logits(x[-1], g, lm_rows, cfg.rms_eps)
        p, r, c = confidence(z)
        logits.append(z)
        probs.append(p)
        verdict.append(r)
        conf.append(c)
    conf = np.asarray(conf, dtype=np.float64)
    return dict(logits=np.asarray(logits), probs=np.asarray(probs), conf=conf,
                verdict=np.asarray(verdict, dtype=np.int32), accept=gate(conf, taus),
                traces=np.asarray(which, dtype=np.int32))


def prefix_pass(cfg, model, prefix_ids: Sequence[np.ndarray]):
    """Dense caches from running each trace's context tokens from position 0.

    Returns (k_dense, v_dense) with k_dense[l][b]: [L_b, Hkv, hd] rotated keys.
    Used by tests to build a cache whose contents are a real prefix pass, so that
    cached suffix prefill can be compared with a full recompute.
    """
    empty = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    traces = [dict(ids=ids, L=0, k_prefix=lambda l: empty, v_prefix=lambda l: empty)
              for ids in prefix_ids]
    _, kvs = forward(cfg, model, traces, keep_kv=True)
    k_dense = [[kvs[b][l][0] for b in range(len(traces))] for l in range(cfg.n_layers)]
    v_dense = [[kvs[b][l][1] for b in range(len(traces))] for l in range(cfg.n_layers)]
    return k_dense, v_dense


def append_rows(cfg, model, kv, block_size: int, suffix_ids, cu_suffix, prefix_lens, n_append: Sequence[int],
                trace_subset: Optional[Sequence[int]] = None) -> dict:
    """Keys and values that join the context when the first n_append[b] suffix tokens of trace b are
    accepted (Algorithm 1, Stage 3: context <- context + accepted draft steps).

    They are the keys (rotated to positions L_b .. L_b + n_append[b] - 1) and values the pass itself
    computes for those tokens in every layer, on top of the cached context; logical row L_b + t of
    trace b receives the pair of suffix token t.
    Returns dict(traces, k, v) with k[l][i], v[l][i]: [n_append[b_i], Hkv, hd] for the i-th listed trace.
    """
    suffix_ids = np.asarray(suffix_ids)
    cu = np.asarray(cu_suffix, dtype=np.int64)
    Ls = np.asarray(prefix_lens, dtype=np.int64)
    which = list(range(len(Ls))) if trace_subset is None else list(trace_subset)
    traces = []
    for b in which:
        L = int(Ls[b])
        n = int(n_append[b])
        if n < 0 or n > cu[b + 1] - cu[b]:
            raise ValueError(f"n_append[{b}] = {n} outside [0, S_b]")
        blk_ids = np.asarray(kv.block_table[b][:(L + block_size - 1) // block_size], dtype=np.int64)
        empty = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))

        def k_prefix(l, blk_ids=blk_ids, L=L):
            return gather_prefix(kv.k_blocks(l, blk_ids), L) if L else empty

        def v_prefix(l, blk_ids=blk_ids, L=L):
            return gather_prefix(kv.v_blocks(l, blk_ids), L) if L else empty

        # only the accepted tokens are run: causal attention makes them independent of what follows
        traces.append(dict(ids=suffix_ids[cu[b]:cu[b] + n], L=L, k_prefix=k_prefix, v_prefix=v_prefix))
    _, kvs = forward(cfg, model, traces, keep_kv=True)
    return dict(traces=np.asarray(which, dtype=np.int32),
                k=[[kvs[i][l][0] for i in range(len(which))] for l in range(cfg.n_layers)],
                v=[[kvs[i][l][1] for i in range(len(which))] for l in range(cfg.n_layers)])


# --------------------------------------------------------------------------- #
# Generation (Algorithm 1: the generate calls of both models) and the
# full-vocabulary reading of the confidence
# --------------------------------------------------------------------------- #
def head_stats(x_last: np.ndarray, final_norm: np.ndarray, lm_head: np.ndarray, eps: float, want_margin: bool = False):
    """(token, max_logit, lse) at one position: z = W_lm . RMSNorm(x_last) over the whole vocabulary,
    token = argmax z (lowest index on ties), lse = log sum_v exp z_v.  The probability of any token v under
    the full softmax is exp(z_v - lse).  With want_margin a fourth value: max_logit minus the second largest
    logit (how clearly the arg max is decided; for tests)."""
    z = np.asarray(lm_head, dtype=np.float64) @ rmsnorm(x_last, final_norm, eps)
    tok = int(np.argmax(z))
    zmax = float(z[tok])
    out = (tok, zmax, zmax + math.log(float(np.sum(np.exp(z - zmax)))))
    if want_margin:
        out += (zmax - float(np.max(np.delete(z, tok))),)
    return out


def next_token(cfg, model, kv, block_size: int, suffix_ids, cu_suffix, prefix_lens,
               verdict_ids: Optional[Sequence[int]] = None, trace_subset: Optional[Sequence[int]] = None) -> dict:
    """Greedy next token after the last suffix position of every listed trace, with the statistics of the
    full-vocabulary softmax.  With verdict_ids it also returns conf_full: the largest full-vocabulary
    probability among the verdict tokens (the other reading of "the corresponding softmax probability"
    after Eq. 3; the restricted confidence is this value renormalised over the verdict tokens).
    model needs lm_head_full() -> [V, d]."""
    suffix_ids = np.asarray(suffix_ids)
    cu = np.asarray(cu_suffix, dtype=np.int64)
    Ls = np.asarray(prefix_lens, dtype=np.int64)
    which = list(range(len(Ls))) if trace_subset is None else list(trace_subset)
    empty = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    traces = []
    for b in which:
        L = int(Ls[b])
        blk_ids = np.asarray(kv.block_table[b][:(L + block_size - 1) // block_size], dtype=np.int64)
        traces.append(dict(ids=suffix_ids[cu[b]:cu[b + 1]], L=L,
                           k_prefix=lambda l, blk_ids=blk_ids, L=L: gather_prefix(kv.k_blocks(l, blk_ids), L) if L else empty,
                           v_prefix=lambda l, blk_ids=blk_ids, L=L: gather_prefix(kv.v_blocks(l, blk_ids), L) if L else empty))
    xs, _ = forward(cfg, model, traces)
    g = np.asarray(model.final_norm, dtype=np.float64)
    head = np.asarray(model.lm_head_full(), dtype=np.float64)
    tok, zmax, lse, conf_full, margin = [], [], [], [], []
    for x in xs:
        t, m, s, mg = head_stats(x[-1], g, head, cfg.rms_eps, want_margin=True)
        tok.append(t); zmax.append(m); lse.append(s); margin.append(mg)
        if verdict_ids is not None:
            zv = verdict_logits(x[-1], g, head[np.asarray(verdict_ids)], cfg.rms_eps)
            conf_full.append(float(np.exp(np.max(zv) - s)))
    out = dict(traces=np.asarray(which, dtype=np.int32), token=np.asarray(tok, dtype=np.int64),
               max_logit=np.asarray(zmax), lse=np.asarray(lse), margin=np.asarray(margin))
    if verdict_ids is not None:
        out["conf_full"] = np.asarray(conf_full)
    return out


def generate_greedy(cfg, model, k_ctx, v_ctx, first_ids: Sequence[int], n_steps: int, want_margin: bool = False):
    """n_steps greedy tokens per trace, one position at a time on a growing context.

    k_ctx[l][b], v_ctx[l][b]: [L_b, Hkv, hd] cached context of trace b; first_ids[b]: the token at position L_b
    (the last token so far, whose keys / values are not cached yet).  Each step runs that one token through the
    layers on top of the cache, appends its keys / values to the context, and takes the arg max of the
    full-vocabulary logits as the next token.
    Returns (tokens [B, n_steps], max_logit, lse, k_ctx, v_ctx) with the grown contexts (each L_b + n_steps rows);
    with want_margin a sixth value, the arg max's lead over the second largest logit at every step."""
    B = len(first_ids)
    k = [[np.asarray(k_ctx[l][b], dtype=np.float64) for b in range(B)] for l in range(cfg.n_layers)]
    v = [[np.asarray(v_ctx[l][b], dtype=np.float64) for b in range(B)] for l in range(cfg.n_layers)]
    g = np.asarray(model.final_norm, dtype=np.float64)
    head = np.asarray(model.lm_head_full(), dtype=np.float64)
    cur = [int(t) for t in first_ids]
    toks = np.zeros((B, n_steps), dtype=np.int64)
    zmax, lse, margin = np.zeros((B, n_steps)), np.zeros((B, n_steps)), np.zeros((B, n_steps))
    for i in range(n_steps):
        traces = [dict(ids=np.asarray([cur[b]]), L=k[0][b].shape[0], k_prefix=lambda l, b=b: k[l][b],
                       v_prefix=lambda l, b=b: v[l][b]) for b in range(B)]
        xs, kvs = forward(cfg, model, traces, keep_kv=True)
        for b in range(B):
            for l in range(cfg.n_layers):
                k[l][b] = np.concatenate([k[l][b], kvs[b][l][0]])
                v[l][b] = np.concatenate([v[l][b], kvs[b][l][1]])
            toks[b, i], zmax[b, i], lse[b, i], margin[b, i] = head_stats(xs[b][-1], g, head, cfg.rms_eps, want_margin=True)
            cur[b] = int(toks[b, i])
    return (toks, zmax, lse, k, v, margin) if want_margin else (toks, zmax, lse, k, v)


# --------------------------------------------------------------------------- #
# Two-tier cascade over the k drafted steps of one request (Algorithm 1, Stage 2;
# Section 4.2, "Cascaded Decision Rule", Eq. 4)
# --------------------------------------------------------------------------- #
NOT_REACHED = -1


def cascade_request(draft_verdict: Sequence[int], draft_conf: Sequence[float], target_verdict, gamma: float,
                    accept_index: int = 0):
    """Cascaded verification of the k drafted steps of one request.

    Written from the definitions rather than as a loop with a counter: Eq. 4 defines the cascaded decision
    V_j of a step as a function of the step alone (the small model's decision where its confidence reaches
    gamma, the large model's otherwise), and the number of accepted steps m is the length of the longest
    run of accepted steps from the start (Section 4.2: steps are accepted up to the first rejection).

    draft_verdict[j], draft_conf[j]: the small model's decision on step j and its confidence.
    target_verdict: callable j -> the large model's decision on step j.  It is expensive, so V_j is
    evaluated on demand and the search for the first rejection goes in step order: the callable is
    invoked exactly for the low-confidence steps up to and including the first rejection, in order,
    once each.
    Returns (m, decision, escalated): decision[j] = V_j for the steps up to and including the first
    rejection, NOT_REACHED after that; escalated[j] = 1 where the large model was consulted.
    """
    k = len(draft_verdict)
    kept = [float(draft_conf[j]) >= float(gamma) for j in range(k)]       # Eq. 4: which case applies to step j
    asked = {}

    def V(j):                                                            # Eq. 4
        if kept[j]:
            return int(draft_verdict[j])
        if j not in asked:
            asked[j] = int(target_verdict(j))
        return asked[j]

    m = next((j for j in range(k) if V(j) != accept_index), k)           # first rejected step; k if none
    looked_at = min(m + 1, k)
    decision = [V(j) if j < looked_at else NOT_REACHED for j in range(k)]
    escalated = [int(j < looked_at and not kept[j]) for j in range(k)]
    return m, decision, escalated


def tree_request(parent: Sequence[int], draft_verdict: Sequence[int], draft_conf: Sequence[float], target, gamma: float,
                 accept_index: int = 0):
    """Tree-structured drafting for one request (Section 4.3, Eq. 5).

    Node j is a candidate step; parent[j] is the node it continues (an earlier index), -1 for a candidate
    of the first layer.  Layer by layer, cascaded verification (Eq. 4) is applied to every candidate that
    continues the step chosen so far; among those that pass, the one with the highest confidence - the
    small model's where its decision was kept, the large model's where it was consulted - is chosen and
    the walk goes on with its children.  It ends at a layer where nothing passes (or at a leaf).
    target: callable j -> (decision, confidence) of the large model, called only for candidates of a
    reached layer whose small-model confidence is below gamma.  Ties go to the lowest index.
    Returns (path, decision, escalated, conf_used): the chosen nodes in order; per node the cascaded
    decision (NOT_REACHED for nodes of layers the walk never looked at), whether the large model was
    consulted, and the confidence that entered the selection (NaN if not reached).
    """
    n = len(parent)
    decision = [NOT_REACHED] * n
    escalated = [0] * n
    conf_used = [float("nan")] * n
    path = []
    cur = -1
    while True:
        layer = [j for j in range(n) if parent[j] == cur]
        if not layer:
            break
        best = None
        for j in layer:
            if draft_conf[j] >= gamma:
                v, p = int(draft_verdict[j]), float(draft_conf[j])
            else:
                v, p = target(j)
                v, p = int(v), float(p)
                escalated[j] = 1
            decision[j], conf_used[j] = v, p
            if v == accept_index and (best is None or p > conf_used[best]):
                best = j
        if best is None:
            break
        path.append(best)
        cur = best
    return path, decision, escalated, conf_used


def cascade_verify(draft, target, block_size: int, suffix_ids, cu_suffix, prefix_lens, verdict_ids, gamma: float,
                   req_start: Sequence[int], request_subset: Optional[Sequence[int]] = None,
                   parent: Optional[Sequence[int]] = None) -> dict:
    """Cascade over a batch of requests.  draft / target: dicts with cfg, model, kv (each model has its
    own cache of the same contexts).  Traces req_start[r] .. req_start[r+1]-1 are the drafted steps of
    request r in order.  The large model's pass runs only for the steps the loop escalates.
    request_subset: evaluate these requests only (requests are independent); the entries of all other
    requests and traces stay NaN / NOT_REACHED.
    parent (tree-structured drafting, Section 4.3): parent[b] = the trace that candidate b continues (a batch
    index inside the same request, smaller than b), -1 for first-layer candidates; then the result also has
    selected [B] (1 on the chosen path), conf_used [B], and accepted_steps is the length of the chosen path."""
    B = len(prefix_lens)
    R = len(req_start) - 1
    which = list(range(R)) if request_subset is None else [int(r) for r in request_subset]
    tr = [b for r in which for b in range(int(req_start[r]), int(req_start[r + 1]))]
    d = verify(draft["cfg"], draft["model"], draft["kv"], block_size, suffix_ids, cu_suffix, prefix_lens, verdict_ids,
               [gamma], trace_subset=tr)
    nv = len(verdict_ids)
    conf_d, verdict_d, logits_d = np.full(B, np.nan), np.full(B, NOT_REACHED, dtype=np.int64), np.full((B, nv), np.nan)
    conf_d[tr], verdict_d[tr], logits_d[tr] = d["conf"], d["verdict"], d["logits"]
    conf_t = np.full(B, np.nan)
    verdict_t = np.full(B, NOT_REACHED, dtype=np.int64)
    logits_t = np.full((B, nv), np.nan)

    def ask_target(b):
        t = verify(target["cfg"], target["model"], target["kv"], block_size, suffix_ids, cu_suffix, prefix_lens,
                   verdict_ids, [gamma], trace_subset=[b])
        conf_t[b], verdict_t[b], logits_t[b] = t["conf"][0], t["verdict"][0], t["logits"][0]
        return int(t["verdict"][0])

    m = np.full(R, NOT_REACHED, dtype=np.int64)
    decision = np.full(B, NOT_REACHED, dtype=np.int64)
    escalated = np.zeros(B, dtype=np.uint8)
    selected = np.zeros(B, dtype=np.uint8)
    conf_used = np.full(B, np.nan)
    for r in which:
        lo, hi = int(req_start[r]), int(req_start[r + 1])
        if parent is None:
            m[r], dec, esc = cascade_request(verdict_d[lo:hi], conf_d[lo:hi], lambda j, lo=lo: ask_target(lo + j), gamma)
        else:
            local = [int(parent[b]) - lo if parent[b] >= 0 else -1 for b in range(lo, hi)]
            path, dec, esc, used = tree_request(local, verdict_d[lo:hi], conf_d[lo:hi],
                                                lambda j, lo=lo: (ask_target(lo + j), conf_t[lo + j]), gamma)
            m[r] = len(path)
            selected[[lo + j for j in path]] = 1
            conf_used[lo:hi] = used
        decision[lo:hi] = dec
        escalated[lo:hi] = esc
    out = dict(accepted_steps=m, decision=decision, escalated=escalated, conf_draft=conf_d, verdict_draft=verdict_d,
               logits_draft=logits_d, conf_target=conf_t, verdict_target=verdict_t, logits_target=logits_t)
    if parent is not None:
        out.update(selected=selected, conf_used=conf_used)
    return out
