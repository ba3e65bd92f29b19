"""Pins for the CPU oracle: brute force on tiny inputs, closed forms, invariants.

None of these compares the oracle with itself through the same formula: each
one checks it against something the mathematics fixes independently.
"""
import math
import os

import numpy as np
import pytest

from oracle import confspec_oracle as O
from tests import brute_force as BF
from tests.helpers import DenseKV, DictModel, small_cfg

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _empty(cfg):
    return np.zeros((0, cfg.n_kv_heads, cfg.head_dim))


def _full_recompute(cfg, model, ids):
    """Oracle over a whole sequence from position 0 (no cache)."""
    e = _empty(cfg)
    xs, kvs = O.forward(cfg, model, [dict(ids=ids, L=0, k_prefix=lambda l: e, v_prefix=lambda l: e)],
                        keep_kv=True)
    return xs[0], kvs[0]


# --------------------------------------------------------------------------- #
# brute force on tiny inputs
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("L,S,hq,hkv", [(3, 3, 2, 1), (0, 4, 2, 2), (5, 1, 4, 2)])
def test_layer_matches_brute_force(L, S, hq, hkv):
    cfg = small_cfg(n_q_heads=hq, n_kv_heads=hkv, rope_theta=50.0)
    model = DictModel(cfg, seed=L * 10 + S)
    rng = np.random.default_rng(7)
    x = rng.normal(0, 1, (S, cfg.d_model))
    kp = rng.normal(0, 1, (L, hkv, cfg.head_dim))
    vp = rng.normal(0, 1, (L, hkv, cfg.head_dim))
    pos = L + np.arange(S)
    got = O.decoder_layer(x, pos, model.layer(0), kp, vp, cfg)
    want = BF.layer(x, L, model.layer(0), kp, vp, cfg)
    for g, w in zip(got, want):
        np.testing.assert_allclose(g, w, rtol=0, atol=1e-12)


def test_whole_pass_matches_brute_force():
    cfg = small_cfg(n_layers=2, n_q_heads=4, n_kv_heads=2, d_model=8, head_dim=2, rope_theta=100.0)
    model = DictModel(cfg, seed=3)
    rng = np.random.default_rng(11)
    L, S = 4, 3
    kd = [[rng.normal(0, 1, (L, 2, 2))] for _ in range(2)]
    vd = [[rng.normal(0, 1, (L, 2, 2))] for _ in range(2)]
    kv = DenseKV(kd, vd, [L], 4, 2, 2)
    ids = np.array([5, 9, 1])
    vids = np.array([7, 2])
    res = O.verify(cfg, model, kv, 4, ids, [0, S], [L], vids, [0.6])
    x = model.embed_rows(ids)
    for l in range(2):
        x, _, _ = BF.layer(x, L, model.layer(l), kd[l][0], vd[l][0], cfg)
    z, p, r, conf = BF.verdict(x[-1], model.final_norm, model.lm_head_rows(vids), cfg.rms_eps)
    np.testing.assert_allclose(res["logits"][0], z, atol=1e-12)
    np.testing.assert_allclose(res["probs"][0], p, atol=1e-12)
    assert res["verdict"][0] == r
    assert abs(res["conf"][0] - conf) < 1e-12
    assert res["accept"][0, 0] == int(conf >= 0.6)


MUTATIONS = {
    "rope_sign": ("rope", lambda a, pos, th: O_rope_orig(a, -np.asarray(pos), th)),
    "rope_identity": ("rope", lambda a, pos, th: a),
    "silu_sigmoid_only": ("silu", lambda z: 1.0 / (1.0 + np.exp(-z))),
    "norm_no_gain": ("rmsnorm", lambda x, g, eps: x / np.sqrt(np.mean(x * x, -1, keepdims=True) + eps)),
    "norm_no_mean": ("rmsnorm", lambda x, g, eps: x / np.sqrt(np.sum(x * x, -1, keepdims=True) + eps) * g),
}
O_rope_orig = O.rope


@pytest.mark.parametrize("name", sorted(MUTATIONS))
def test_planted_mistakes_are_caught_by_brute_force(name, monkeypatch):
    """A wrong sign, a dropped gain or a wrong activation in the oracle fails the pin."""
    attr, repl = MUTATIONS[name]
    monkeypatch.setattr(O, attr, repl)
    cfg = small_cfg(rope_theta=50.0)
    model = DictModel(cfg, seed=1)
    rng = np.random.default_rng(2)
    L, S = 3, 3
    x = rng.normal(0, 1, (S, cfg.d_model))
    kp = rng.normal(0, 1, (L, 1, cfg.head_dim))
    vp = rng.normal(0, 1, (L, 1, cfg.head_dim))
    got = O.decoder_layer(x, L + np.arange(S), model.layer(0), kp, vp, cfg)[0]
    want = BF.layer(x, L, model.layer(0), kp, vp, cfg)[0]
    assert np.max(np.abs(got - want)) > 1e-6


def test_planted_gqa_and_mask_mistakes_are_caught(monkeypatch):
    cfg = small_cfg(n_q_heads=4, n_kv_heads=2, rope_theta=50.0)
    rng = np.random.default_rng(5)
    L, S = 2, 3
    q = rng.normal(0, 1, (S, 4, 4))
    k = rng.normal(0, 1, (L + S, 2, 4))
    v = rng.normal(0, 1, (L + S, 2, 4))
    good = O.attention(q, k, v, L)
    # head i reading kv head i % Hkv instead of i // G
    wrong_map = np.stack([O.attention(q[:, [i]], k[:, [i % 2]], v[:, [i % 2]], L)[:, 0] for i in range(4)], 1)
    assert np.max(np.abs(good - wrong_map)) > 1e-3
    # off-by-one causal horizon
    assert np.max(np.abs(good - O.attention(q, k, v, L + 1))) > 1e-3
    assert np.max(np.abs(good - O.attention(q, k, v, L - 1))) > 1e-3


# --------------------------------------------------------------------------- #
# KV caching, positions, block table
# --------------------------------------------------------------------------- #
def test_cached_suffix_prefill_equals_full_recompute():
    cfg = small_cfg(n_layers=3, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=4, d_ffn=24, vocab=31)
    model = DictModel(cfg, seed=4)
    rng = np.random.default_rng(9)
    Ls, Ss = [6, 0, 11], [4, 5, 1]
    pre = [rng.integers(0, cfg.vocab, L) for L in Ls]
    suf = [rng.integers(0, cfg.vocab, S) for S in Ss]
    kd, vd = O.prefix_pass(cfg, model, pre)
    kv = DenseKV(kd, vd, Ls, 4, 2, 4, perm_seed=1)
    cu = np.concatenate([[0], np.cumsum(Ss)])
    vids = [3, 17]
    res = O.verify(cfg, model, kv, 4, np.concatenate(suf), cu, Ls, vids, [0.5])
    for b in range(3):
        x, _ = _full_recompute(cfg, model, np.concatenate([pre[b], suf[b]]))
        z = O.verdict_logits(x[-1], model.final_norm, model.lm_head_rows(vids), cfg.rms_eps)
        np.testing.assert_allclose(res["logits"][b], z, rtol=0, atol=1e-11)


def test_block_permutation_leaves_outputs_bit_identical():
    cfg = small_cfg(n_layers=2)
    model = DictModel(cfg, seed=6)
    rng = np.random.default_rng(1)
    Ls, Ss = [9, 5], [2, 3]
    kd = [[rng.normal(0, 1, (L, 1, 4)) for L in Ls] for _ in range(2)]
    vd = [[rng.normal(0, 1, (L, 1, 4)) for L in Ls] for _ in range(2)]
    ids = rng.integers(0, cfg.vocab, sum(Ss))
    outs = []
    for perm_seed in (0, 1, 2):
        kv = DenseKV(kd, vd, Ls, 4, 1, 4, perm_seed=perm_seed)
        outs.append(O.verify(cfg, model, kv, 4, ids, [0, 2, 5], Ls, [1, 2], [0.7])["logits"])
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


def test_gather_prefix_reads_block_then_slot():
    blocks = np.arange(3 * 2 * 4 * 5, dtype=np.float64).reshape(3, 2, 4, 5)
    rows = O.gather_prefix(blocks, 10)
    want = blocks.transpose(0, 2, 1, 3).reshape(12, 2, 5)[:10]
    assert np.array_equal(rows, want)
    assert rows[6, 1, 2] == blocks[1, 1, 2, 2]


def test_padding_slots_of_the_last_block_are_never_read():
    cfg = small_cfg(n_layers=1)
    model = DictModel(cfg, seed=8)
    rng = np.random.default_rng(3)
    kd = [[rng.normal(0, 1, (5, 1, 4))]]
    vd = [[rng.normal(0, 1, (5, 1, 4))]]
    kv = DenseKV(kd, vd, [5], 4, 1, 4)   # slots 5..7 of the second block hold a 1e30 poison
    z = O.verify(cfg, model, kv, 4, [1, 2], [0, 2], [5], [0, 1], [0.5])["logits"]
    assert np.all(np.abs(z) < 1e6)


# --------------------------------------------------------------------------- #
# rotary embedding
# --------------------------------------------------------------------------- #
def test_rope_is_identity_at_position_zero_and_a_rotation_elsewhere():
    rng = np.random.default_rng(0)
    a = rng.normal(0, 1, (3, 2, 8))
    assert np.array_equal(O.rope(a, np.zeros(3), 1e4), a)
    b = O.rope(a, np.array([1, 7, 1000]), 1e4)
    np.testing.assert_allclose(np.sum(b * b, -1), np.sum(a * a, -1), rtol=1e-13)
    # first pair of dims rotates by exactly `pos` radians (frequency theta^0 = 1)
    ang = 7.0
    np.testing.assert_allclose(b[1, 0, 0], a[1, 0, 0] * math.cos(ang) - a[1, 0, 4] * math.sin(ang), atol=1e-13)
    np.testing.assert_allclose(b[1, 0, 4], a[1, 0, 4] * math.cos(ang) + a[1, 0, 0] * math.sin(ang), atol=1e-13)
    # last pair uses frequency theta^(-2*(hd/2-1)/hd)
    ang = 1000.0 * 1e4 ** (-6.0 / 8.0)
    np.testing.assert_allclose(b[2, 1, 3], a[2, 1, 3] * math.cos(ang) - a[2, 1, 7] * math.sin(ang), atol=1e-12)


def test_rope_relative_position_property_under_full_recompute():
    """Shifting every position by a constant leaves attention outputs unchanged."""
    cfg = small_cfg(n_layers=2, rope_theta=1e4)
    model = DictModel(cfg, seed=12)
    ids = np.array([3, 1, 4, 1, 5, 9])
    e = _empty(cfg)
    x0 = model.embed_rows(ids)
    outs = []
    for shift in (0, 37):
        x = x0
        for l in range(cfg.n_layers):
            x, _, _ = O.decoder_layer(x, shift + np.arange(len(ids)), model.layer(l), e, e, cfg)
        outs.append(x)
    np.testing.assert_allclose(outs[0], outs[1], rtol=0, atol=1e-10)


# --------------------------------------------------------------------------- #
# attention closed forms
# --------------------------------------------------------------------------- #
def test_zero_queries_give_running_mean_of_values():
    rng = np.random.default_rng(4)
    L, S = 5, 4
    q = np.zeros((S, 2, 4))
    k = rng.normal(0, 1, (L + S, 1, 4))
    v = rng.normal(0, 1, (L + S, 1, 4))
    o = O.attention(q, k, v, L)
    for t in range(S):
        want = v[: L + t + 1, 0].mean(axis=0)
        np.testing.assert_allclose(o[t, 0], want, atol=1e-14)
        np.testing.assert_allclose(o[t, 1], want, atol=1e-14)


def test_single_token_attends_to_itself_only():
    rng = np.random.default_rng(5)
    q = rng.normal(0, 1, (1, 2, 4))
    k = rng.normal(0, 1, (1, 2, 4))
    v = rng.normal(0, 1, (1, 2, 4))
    np.testing.assert_allclose(O.attention(q, k, v, 0)[0], v[0], atol=1e-15)


def test_attention_scale_is_inverse_sqrt_head_dim():
    """Two keys, one query: weights follow exp(q.k / sqrt(hd)) exactly."""
    q = np.array([[[2.0, 0.0, 0.0, 0.0]]])
    k = np.array([[[1.0, 0, 0, 0]], [[3.0, 0, 0, 0]]])
    v = np.array([[[1.0, 0, 0, 0]], [[0.0, 1, 0, 0]]])
    o = O.attention(q, k, v, 1)[0, 0]
    w1 = math.exp(6.0 / 2.0) / (math.exp(2.0 / 2.0) + math.exp(6.0 / 2.0))
    np.testing.assert_allclose(o[:2], [1 - w1, w1], atol=1e-15)


def test_softmax_shift_invariance_and_normalisation():
    rng = np.random.default_rng(6)
    s = rng.normal(0, 3, (4, 9))
    p = O.softmax(s)
    np.testing.assert_allclose(p.sum(-1), 1.0, atol=1e-15)
    np.testing.assert_allclose(O.softmax(s + 123.0), p, atol=1e-13)
    np.testing.assert_allclose(p[0], np.exp(s[0]) / np.exp(s[0]).sum(), atol=1e-15)


# --------------------------------------------------------------------------- #
# residual / MLP special cases
# --------------------------------------------------------------------------- #
def test_zero_output_projections_make_layers_the_identity():
    cfg = small_cfg(n_layers=3)
    model = DictModel(cfg, seed=13)
    for lw in model.layers:
        lw["wo"] = np.zeros_like(lw["wo"])
        lw["wd"] = np.zeros_like(lw["wd"])
    ids = np.array([4, 8, 15])
    kd = [[np.ones((2, 1, 4))] for _ in range(3)]
    kv = DenseKV(kd, kd, [2], 4, 1, 4)
    vids = [16, 20]
    res = O.verify(cfg, model, kv, 4, ids, [0, 3], [2], vids, [0.5])
    x = model.embed[15]
    y = x / math.sqrt(float(np.mean(x * x)) + cfg.rms_eps) * model.final_norm
    want = model.lm_head[vids] @ y
    np.testing.assert_allclose(res["logits"][0], want, atol=1e-13)


def test_silu_and_mlp_closed_form_single_unit():
    cfg = small_cfg(n_layers=1, d_model=2, n_q_heads=1, n_kv_heads=1, head_dim=2, d_ffn=1)
    lw = dict(attn_norm=np.ones(2), wq=np.zeros((2, 2)), wk=np.zeros((2, 2)), wv=np.zeros((2, 2)),
              wo=np.zeros((2, 2)), mlp_norm=np.array([1.0, 1.0]),
              wg=np.array([[1.0, 0.0]]), wu=np.array([[0.0, 1.0]]), wd=np.array([[1.0], [-2.0]]))
    x = np.array([[3.0, 4.0]])
    out, _, _ = O.decoder_layer(x, np.array([0]), lw, np.zeros((0, 1, 2)), np.zeros((0, 1, 2)), cfg)
    r = math.sqrt((9 + 16) / 2 + cfg.rms_eps)
    g, u = 3.0 / r, 4.0 / r
    act = g / (1 + math.exp(-g)) * u
    np.testing.assert_allclose(out[0], [3.0 + act, 4.0 - 2 * act], atol=1e-14)


# --------------------------------------------------------------------------- #
# verdict head, confidence, gate
# --------------------------------------------------------------------------- #
def test_restricted_softmax_equals_renormalised_full_vocab_softmax():
    cfg = small_cfg(vocab=257, d_model=16)
    model = DictModel(cfg, seed=21, std=0.5)
    rng = np.random.default_rng(2)
    x_last = rng.normal(0, 1, cfg.d_model)
    vids = np.array([200, 3, 77])
    z = O.verdict_logits(x_last, model.final_norm, model.lm_head_rows(vids), cfg.rms_eps)
    p, r, conf = O.confidence(z)
    y = x_last / np.sqrt(np.mean(x_last ** 2) + cfg.rms_eps) * model.final_norm
    full = model.lm_head @ y                      # the whole LM head
    pf = np.exp(full - full.max())
    pf /= pf.sum()
    np.testing.assert_allclose(z, full[vids], atol=1e-13)
    np.testing.assert_allclose(p, pf[vids] / pf[vids].sum(), atol=1e-13)
    assert r == int(np.argmax(pf[vids]))


def test_two_verdict_confidence_is_sigmoid_of_logit_gap():
    rng = np.random.default_rng(3)
    for _ in range(50):
        z = rng.normal(0, 3, 2)
        p, r, conf = O.confidence(z)
        assert abs(conf - 1 / (1 + math.exp(-abs(z[0] - z[1])))) < 1e-14
        assert r == (0 if z[0] >= z[1] else 1)
        assert abs(p.sum() - 1) < 1e-15 and 0.5 <= conf <= 1.0


@pytest.mark.parametrize("n", [2, 3, 8])
def test_confidence_bounds_for_n_verdicts(n):
    rng = np.random.default_rng(n)
    for _ in range(20):
        p, r, conf = O.confidence(rng.normal(0, 2, n))
        assert 1.0 / n - 1e-15 <= conf <= 1.0 and abs(p.sum() - 1) < 1e-14 and p[r] == p.max()


def test_gate_golden_closed_form_cases():
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "gate_closed_form.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 7
    taus = [0.8, 0.9, 0.95]
    for r in rows:
        z = np.array([float(r[0]), float(r[1])])
        p, verdict, conf = O.confidence(z)
        assert verdict == int(r[2])
        assert abs(conf - float(r[3])) < 1e-14
        acc = O.gate(np.array([conf]), taus)[:, 0]
        assert list(acc) == [int(v) for v in r[4:7]]


def test_gate_is_non_strict_and_monotone_in_tau():
    conf = np.array([0.5, 0.75, 0.9, 0.9000001, 1.0])
    acc = O.gate(conf, [0.0, 0.5, 0.9, 0.95, 1.0, 1.0000001])
    assert list(acc[2]) == [0, 0, 1, 1, 1]          # equality accepts (p >= gamma)
    assert acc[0].all() and acc[1].all()            # tau <= 1/n accepts everything
    assert list(acc[4]) == [0, 0, 0, 0, 1] and not acc[5].any()
    for i in range(len(acc) - 1):                   # accept set shrinks as tau rises
        assert np.all(acc[i + 1] <= acc[i])


def test_trace_results_do_not_depend_on_batch_composition():
    cfg = small_cfg(n_layers=2)
    model = DictModel(cfg, seed=30)
    rng = np.random.default_rng(8)
    Ls, Ss = [7, 3, 0], [2, 4, 3]
    kd = [[rng.normal(0, 1, (L, 1, 4)) for L in Ls] for _ in range(2)]
    vd = [[rng.normal(0, 1, (L, 1, 4)) for L in Ls] for _ in range(2)]
    ids = rng.integers(0, cfg.vocab, sum(Ss))
    cu = np.concatenate([[0], np.cumsum(Ss)])
    kv = DenseKV(kd, vd, Ls, 4, 1, 4)
    whole = O.verify(cfg, model, kv, 4, ids, cu, Ls, [1, 2], [0.7])
    for b in range(3):
        alone = O.verify(cfg, model, kv, 4, ids, cu, Ls, [1, 2], [0.7], trace_subset=[b])
        assert np.array_equal(alone["logits"][0], whole["logits"][b])
    # reversed order of traces, re-packed
    order = [2, 0, 1]
    ids2 = np.concatenate([ids[cu[b]:cu[b + 1]] for b in order])
    cu2 = np.concatenate([[0], np.cumsum([Ss[b] for b in order])])
    kv2 = DenseKV([[k[b] for b in order] for k in kd], [[v[b] for b in order] for v in vd],
                  [Ls[b] for b in order], 4, 1, 4, perm_seed=5)
    again = O.verify(cfg, model, kv2, 4, ids2, cu2, [Ls[b] for b in order], [1, 2], [0.7])
    for i, b in enumerate(order):
        assert np.array_equal(again["logits"][i], whole["logits"][b])
