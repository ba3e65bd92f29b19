"""Pins of the oracle's append rows (Algorithm 1, Stage 3: accepted draft steps join the context): a context built
in chunks must be the context of a single pass, and what is appended cannot depend on the tokens after it."""
import numpy as np

from oracle import confspec_oracle as O
from tests.helpers import DenseKV, DictModel, small_cfg


def _setup(seed=5, n_layers=3):
    cfg = small_cfg(n_layers=n_layers, d_model=16, n_q_heads=4, n_kv_heads=2, head_dim=8, d_ffn=24, vocab=37)
    model = DictModel(cfg, seed=seed)
    rng = np.random.default_rng(seed + 1)
    lens = [11, 1, 7, 18]
    toks = [rng.integers(0, cfg.vocab, size=n) for n in lens]
    return cfg, model, toks


def test_context_built_in_chunks_equals_single_pass():
    cfg, model, toks = _setup()
    bs = 4
    k_all, v_all = O.prefix_pass(cfg, model, toks)                     # rows 0 .. n-1 of every trace in one pass
    cut = [5, 0, 7, 9]                                                 # already cached: rows 0 .. cut-1
    k_c = [[k_all[l][b][:cut[b]] for b in range(4)] for l in range(cfg.n_layers)]
    v_c = [[v_all[l][b][:cut[b]] for b in range(4)] for l in range(cfg.n_layers)]
    kv = DenseKV(k_c, v_c, cut, bs, cfg.n_kv_heads, cfg.head_dim, perm_seed=3)
    suffix = [toks[b][cut[b]:] for b in range(4)]                      # trace 2 has nothing left
    suffix[2] = np.array([4, 9], dtype=np.int64)                       # (it still verifies something)
    cu = np.concatenate([[0], np.cumsum([len(s) for s in suffix])])
    n_app = [len(toks[b]) - cut[b] for b in range(4)]
    n_app[2] = 0
    got = O.append_rows(cfg, model, kv, bs, np.concatenate(suffix), cu, cut, n_app)
    for l in range(cfg.n_layers):
        for b in range(4):
            assert got["k"][l][b].shape == (n_app[b], cfg.n_kv_heads, cfg.head_dim)
            assert np.abs(got["k"][l][b] - k_all[l][b][cut[b]:cut[b] + n_app[b]]).max(initial=0.0) < 1e-11
            assert np.abs(got["v"][l][b] - v_all[l][b][cut[b]:cut[b] + n_app[b]]).max(initial=0.0) < 1e-11
    # a plausible slip - new keys rotated as if the chunk started at position 0 - would not survive this comparison
    shifted = O.append_rows(cfg, model, kv, bs, np.concatenate(suffix), cu, [0, 0, 0, 0], n_app)
    assert np.abs(shifted["k"][0][0] - k_all[0][0][cut[0]:]).max() > 1e-3


def test_appended_rows_do_not_depend_on_later_tokens_and_subset_matches():
    cfg, model, toks = _setup(seed=9)
    bs = 4
    k_all, v_all = O.prefix_pass(cfg, model, [t[:6] for t in toks[:1]] + [toks[1][:1]] + [t[:6] for t in toks[2:]])
    cut = [6, 1, 6, 6]
    kv = DenseKV(k_all, v_all, cut, bs, cfg.n_kv_heads, cfg.head_dim, perm_seed=1)
    rng = np.random.default_rng(2)
    suffix_a = [rng.integers(0, cfg.vocab, size=n) for n in (5, 3, 4, 6)]
    n_app = [2, 3, 0, 4]
    suffix_b = [s.copy() for s in suffix_a]
    for b, s in enumerate(suffix_b):
        s[n_app[b]:] = (s[n_app[b]:] + 1) % cfg.vocab                  # change everything after the appended part
    cu = np.concatenate([[0], np.cumsum([len(s) for s in suffix_a])])
    ra = O.append_rows(cfg, model, kv, bs, np.concatenate(suffix_a), cu, cut, n_app)
    rb = O.append_rows(cfg, model, kv, bs, np.concatenate(suffix_b), cu, cut, n_app)
    sub = O.append_rows(cfg, model, kv, bs, np.concatenate(suffix_a), cu, cut, n_app, trace_subset=[3, 0])
    for l in range(cfg.n_layers):
        for b in range(4):
            assert np.array_equal(ra["k"][l][b], rb["k"][l][b]) and np.array_equal(ra["v"][l][b], rb["v"][l][b])
        assert np.array_equal(sub["k"][l][0], ra["k"][l][3]) and np.array_equal(sub["v"][l][1], ra["v"][l][0])
    # the appended rows are what a later pass reads: verifying the rest of the suffix on top of the grown context
    # gives the same residual stream as verifying the whole suffix on the old one
    b = 3
    tr_old = dict(ids=suffix_a[b], L=cut[b], k_prefix=lambda l: k_all[l][b], v_prefix=lambda l: v_all[l][b])
    x_old, _ = O.forward(cfg, model, [tr_old])
    grown_k = [np.concatenate([k_all[l][b], ra["k"][l][b]]) for l in range(cfg.n_layers)]
    grown_v = [np.concatenate([v_all[l][b], ra["v"][l][b]]) for l in range(cfg.n_layers)]
    tr_new = dict(ids=suffix_a[b][n_app[b]:], L=cut[b] + n_app[b], k_prefix=lambda l: grown_k[l],
                  v_prefix=lambda l: grown_v[l])
    x_new, _ = O.forward(cfg, model, [tr_new])
    assert np.abs(x_new[0] - x_old[0][n_app[b]:]).max() < 1e-10


def test_append_rows_rejects_counts_outside_the_suffix():
    cfg, model, toks = _setup()
    k_all, v_all = O.prefix_pass(cfg, model, [t[:4] for t in toks])
    kv = DenseKV(k_all, v_all, [4, 1, 4, 4], 4, cfg.n_kv_heads, cfg.head_dim)
    ids = np.arange(8) % cfg.vocab
    for bad in ([3, 0, 0, 0], [-1, 0, 0, 0]):
        try:
            O.append_rows(cfg, model, kv, 4, ids, [0, 2, 4, 6, 8], [4, 1, 4, 4], bad)
        except ValueError:
            continue
        raise AssertionError("count outside [0, S_b] accepted")
