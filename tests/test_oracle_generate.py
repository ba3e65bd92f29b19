"""Pins of the oracle's generation step and of the full-vocabulary confidence: a library log-sum-exp, the
renormalisation identity between the two readings of the confidence, and greedy generation on a growing cache
against recomputing the whole sequence from position 0 at every step."""
import numpy as np
from scipy.special import logsumexp, softmax as sp_softmax

from oracle import confspec_oracle as O
from tests.helpers import DenseKV, DictModel, small_cfg


def _setup(seed=3):
    cfg = small_cfg(n_layers=2, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=24, vocab=41)
    return cfg, DictModel(cfg, seed=seed)


def test_head_stats_against_library_routines():
    cfg, model = _setup()
    rng = np.random.default_rng(0)
    x = rng.normal(0, 2.0, cfg.d_model)
    tok, zmax, lse = O.head_stats(x, model.final_norm, model.lm_head, cfg.rms_eps)
    z = model.lm_head @ O.rmsnorm(x, model.final_norm, cfg.rms_eps)
    assert tok == int(np.argmax(z)) and abs(zmax - z.max()) < 1e-13 and abs(lse - logsumexp(z)) < 1e-12
    assert abs(np.exp(z - lse).sum() - 1.0) < 1e-12
    # ties: the lowest index wins
    head = model.lm_head.copy()
    head[7] = head[3]
    z2 = head @ O.rmsnorm(x, model.final_norm, cfg.rms_eps)
    if np.argmax(z2) in (3, 7):
        assert O.head_stats(x, model.final_norm, head, cfg.rms_eps)[0] == 3


def test_full_vocabulary_confidence_renormalises_to_the_restricted_one():
    cfg, model = _setup(seed=4)
    toks = [np.array([1, 5, 9, 2, 30]), np.array([7])]
    k, v = O.prefix_pass(cfg, model, [t[:3] for t in toks[:1]] + [toks[1][:0]])
    kv = DenseKV(k, v, [3, 0], 4, cfg.n_kv_heads, cfg.head_dim)
    ids = np.concatenate([toks[0][3:], toks[1]])
    cu = [0, 2, 3]
    vids = [11, 4, 29]
    full = O.next_token(cfg, model, kv, 4, ids, cu, [3, 0], verdict_ids=vids)
    res = O.verify(cfg, model, kv, 4, ids, cu, [3, 0], vids, [0.5])
    p_full = np.exp(res["logits"] - full["lse"][:, None])           # full-vocabulary probabilities of the verdict tokens
    assert np.allclose(p_full.max(axis=1), full["conf_full"], atol=1e-14)
    assert np.allclose(p_full.max(axis=1) / p_full.sum(axis=1), res["conf"], atol=1e-13)
    assert np.all(full["conf_full"] <= res["conf"] + 1e-15)
    # the arg max token and its probability against scipy's softmax on logits from the full head
    for i in range(2):
        x_ids = toks[i]
        xs, _ = O.forward(cfg, model, [dict(ids=x_ids, L=0, k_prefix=lambda l: np.zeros((0, 2, 8)),
                                             v_prefix=lambda l: np.zeros((0, 2, 8)))])
        z = model.lm_head @ O.rmsnorm(xs[0][-1], model.final_norm, cfg.rms_eps)
        assert full["token"][i] == np.argmax(z)
        assert abs(np.exp(full["max_logit"][i] - full["lse"][i]) - sp_softmax(z).max()) < 1e-12


def test_greedy_generation_on_a_growing_cache_equals_recomputing_from_scratch():
    cfg, model = _setup(seed=6)
    ctx = [np.array([3, 1, 4, 1, 5, 9, 2]), np.array([6]), np.array([5, 3, 5, 8])]
    k, v = O.prefix_pass(cfg, model, [c[:-1] for c in ctx])          # everything but the last token is cached
    n = 5
    toks, zmax, lse, k2, v2 = O.generate_greedy(cfg, model, k, v, [c[-1] for c in ctx], n)
    e = np.zeros((0, cfg.n_kv_heads, cfg.head_dim))
    for b, c in enumerate(ctx):
        seq = list(c)
        for i in range(n):
            xs, _ = O.forward(cfg, model, [dict(ids=np.asarray(seq), L=0, k_prefix=lambda l: e, v_prefix=lambda l: e)])
            z = model.lm_head @ O.rmsnorm(xs[0][-1], model.final_norm, cfg.rms_eps)
            assert toks[b, i] == int(np.argmax(z)), (b, i)
            assert abs(lse[b, i] - logsumexp(z)) < 1e-10 and abs(zmax[b, i] - z.max()) < 1e-10
            seq.append(int(toks[b, i]))
        # the grown context is the context of the whole sequence (all but the token generated last)
        k_all, v_all = O.prefix_pass(cfg, model, [np.asarray(seq[:-1])])
        for l in range(cfg.n_layers):
            assert np.abs(k2[l][b] - k_all[l][0]).max() < 1e-10 and np.abs(v2[l][b] - v_all[l][0]).max() < 1e-10
