"""Pins of the oracle's cascade loop (Algorithm 1, Stage 2; Eq. 4): exhaustive enumeration of small requests
against an independently written closed form, and the limiting thresholds."""
import itertools

import numpy as np

from oracle import confspec_oracle as O


def _closed_form(rd, conf, rt, gamma):
    """V_j = r_D where conf >= gamma else r_T; m = length of the leading run of accepts (index 0);
    steps after the first rejection are not reached."""
    rd, conf, rt = np.asarray(rd), np.asarray(conf), np.asarray(rt)
    use_t = conf < gamma
    v = np.where(use_t, rt, rd)
    acc = (v == 0).astype(int)
    m = int(np.cumprod(acc).sum())
    reached = np.arange(len(v)) <= m          # the accepted ones and the first rejection
    return m, np.where(reached, v, O.NOT_REACHED), (use_t & reached).astype(int)


def test_cascade_loop_matches_closed_form_on_every_small_request():
    gamma = 0.9
    for k in range(1, 5):
        for rd in itertools.product((0, 1), repeat=k):
            for hi in itertools.product((0, 1), repeat=k):          # confident or not
                for rt in itertools.product((0, 1), repeat=k):
                    conf = [0.97 if h else 0.61 for h in hi]
                    asked = []
                    m, dec, esc = O.cascade_request(rd, conf, lambda j: (asked.append(j), rt[j])[1], gamma)
                    m2, dec2, esc2 = _closed_form(rd, conf, rt, gamma)
                    assert (m, list(dec), list(esc)) == (m2, list(dec2), list(esc2)), (rd, hi, rt)
                    assert asked == [j for j in range(k) if esc[j]]      # the large model is asked only when consulted


def test_cascade_thresholds_and_equality():
    rd, rt, conf = [0, 1, 0], [1, 0, 0], [0.7, 0.8, 0.9]
    # gamma = 0: the small model always decides; gamma above 1: the large model always decides
    assert O.cascade_request(rd, conf, lambda j: rt[j], 0.0)[:2] == (1, [0, 1, O.NOT_REACHED])
    assert O.cascade_request(rd, conf, lambda j: rt[j], 1.01)[:2] == (0, [1, O.NOT_REACHED, O.NOT_REACHED])
    # confidence equal to the threshold keeps the small model's decision (p >= gamma)
    m, dec, esc = O.cascade_request([0], [0.9], lambda j: 1, 0.9)
    assert (m, dec, esc) == (1, [0], [0])
    m, dec, esc = O.cascade_request([0], [np.nextafter(0.9, 0)], lambda j: 1, 0.9)
    assert (m, dec, esc) == (0, [1], [1])
    # all accepted: m = k; other verdict indices count as rejections
    assert O.cascade_request([0, 0], [1.0, 1.0], lambda j: 1, 0.5)[0] == 2
    assert O.cascade_request([2, 0], [1.0, 1.0], lambda j: 0, 0.5)[0] == 0


def test_cascade_verify_consults_the_large_model_lazily():
    from tests.helpers import small_cfg, DictModel, DenseKV  # noqa: F401  (availability of the helpers)
    import confspec_workloads as W
    wl_d = W.tiny_workload("casc_d", 71, dtype="fp32", n_layers=1, d_model=64, n_q_heads=2, n_kv_heads=1, head_dim=32,
                           d_ffn=128, vocab=97, prefix_lens=(5, 9, 0, 17, 3, 12), suffix_lens=(4, 3, 6, 2, 5, 1))
    wl_t = W.tiny_workload("casc_t", 72, dtype="fp32", n_layers=2, d_model=96, n_q_heads=2, n_kv_heads=2, head_dim=48,
                           d_ffn=160, vocab=97, prefix_lens=wl_d.prefix_lens, suffix_lens=wl_d.suffix_lens)
    batch = W.make_batch(wl_d, "cpu")
    sides = []
    for wl in (wl_d, wl_t):
        weights = W.make_weights(wl.model, wl.seed, "cpu")
        kv = W.make_seeded_kv(wl, batch, "cpu")
        sides.append(dict(cfg=wl.model, model=W.OracleModelView(weights), kv=W.OracleKVView(kv, batch)))
    vids = W.draw_verdict_ids(wl_d)
    ids, cu, pl = batch.suffix_ids.numpy(), batch.h_cu_suffix, batch.h_prefix_lens
    req_start = [0, 2, 3, 6]
    res = {g: O.cascade_verify(sides[0], sides[1], wl_d.block_size, ids, cu, pl, vids, g, req_start) for g in (0.0, 0.55, 2.0)}
    full_t = O.verify(sides[1]["cfg"], sides[1]["model"], sides[1]["kv"], wl_d.block_size, ids, cu, pl, vids, [0.5])
    full_d = O.verify(sides[0]["cfg"], sides[0]["model"], sides[0]["kv"], wl_d.block_size, ids, cu, pl, vids, [0.5])
    for g, r in res.items():
        for q in range(3):
            lo, hi = req_start[q], req_start[q + 1]
            m, dec, esc = _closed_form(full_d["verdict"][lo:hi], full_d["conf"][lo:hi], full_t["verdict"][lo:hi], g)
            assert r["accepted_steps"][q] == m
            assert list(r["decision"][lo:hi]) == list(dec) and list(r["escalated"][lo:hi]) == list(esc)
        asked = ~np.isnan(r["conf_target"])
        assert np.array_equal(asked, r["escalated"].astype(bool))          # no pass of the large model that was not needed
        assert np.allclose(r["conf_target"][asked], full_t["conf"][asked], atol=1e-12)
    assert res[0.0]["escalated"].sum() == 0 and res[2.0]["escalated"].sum() >= 3
    # requests are independent: evaluating a subset of them gives the same entries as the full run
    sub = O.cascade_verify(sides[0], sides[1], wl_d.block_size, ids, cu, pl, vids, 0.55, req_start, request_subset=[2, 0])
    full = res[0.55]
    for q in (0, 2):
        lo, hi = req_start[q], req_start[q + 1]
        assert sub["accepted_steps"][q] == full["accepted_steps"][q]
        for k in ("decision", "escalated", "conf_draft", "verdict_draft", "conf_target", "verdict_target"):
            assert np.array_equal(sub[k][lo:hi], full[k][lo:hi], equal_nan=True), k
    assert sub["accepted_steps"][1] == O.NOT_REACHED and np.isnan(sub["conf_draft"][2])
